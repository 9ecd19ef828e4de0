"""Backward pass of the expert FFN -- TEST INFRASTRUCTURE ONLY (numpy, float64).

Section 2.1 of the paper: training repeats the dispatch -> compute -> combine exchange of the forward pass for the
gradients (the all-to-alls of the backward pass), so the receiving rank also runs the expert computation backwards on the
rows each matching delivers.  For the SwiGLU expert of oracle/ffn.py,

    g = x Wg^T,  u = x Wu^T,  s = g * sigmoid(g),  h = s * u,  y = h Wd^T,

the chain rule gives, for the gradient dy of a scalar loss with respect to y,

    dh = dy Wd
    du = dh * s
    dg = dh * u * sigmoid(g) * (1 + g * (1 - sigmoid(g)))          (the derivative of g * sigmoid(g))
    dx = dg Wg + du Wu
    dWd_e = sum over the rows m of expert e of  dy[m]^T h[m]        [d][f]
    dWg_e = sum_m dg[m]^T x[m],   dWu_e = sum_m du[m]^T x[m]        [f][d]

written out below in float64, one expert at a time, from the same input bits the GPU gets.
"""
from __future__ import annotations

import numpy as np

from .ffn import decode_bf16


def expert_ffn_backward_sliced(x_bits: np.ndarray, dy_bits: np.ndarray, offsets: np.ndarray, E_loc: int, weights):
    """x_bits, dy_bits uint16 [M][d] (bf16 bit patterns); offsets int32 [S*E_loc+1] (group g = slice*E_loc + expert);
    weights: bf16 FFNWeights.  Returns (dx float64 [M_used][d], dWg [E_loc][f][d], dWu [E_loc][f][d], dWd [E_loc][d][f])."""
    assert weights.dtype == "bf16"
    offsets = np.asarray(offsets, dtype=np.int64)
    M_used = int(offsets[-1])
    d = x_bits.shape[1]
    f = weights.w_gate.shape[1]
    G = len(offsets) - 1
    assert G % E_loc == 0
    rows = np.arange(M_used, dtype=np.int64)
    expert_of_row = (np.searchsorted(offsets, rows, side="right") - 1) % E_loc
    dx = np.zeros((M_used, d), dtype=np.float64)
    dWg = np.zeros((E_loc, f, d), dtype=np.float64)
    dWu = np.zeros((E_loc, f, d), dtype=np.float64)
    dWd = np.zeros((E_loc, d, f), dtype=np.float64)
    for e in range(E_loc):
        sel = np.flatnonzero(expert_of_row == e)
        if sel.size == 0:
            continue
        Wg, Wu, Wd = decode_bf16(weights.w_gate[e]), decode_bf16(weights.w_up[e]), decode_bf16(weights.w_down[e])
        x = decode_bf16(x_bits[sel])
        dy = decode_bf16(dy_bits[sel])
        g = x @ Wg.T
        u = x @ Wu.T
        sig = 1.0 / (1.0 + np.exp(-g))
        s = g * sig
        h = s * u
        dh = dy @ Wd
        du = dh * s
        dg = dh * u * sig * (1.0 + g * (1.0 - sig))
        dx[sel] = dg @ Wg + du @ Wu
        dWd[e] = dy.T @ h
        dWg[e] = dg.T @ x
        dWu[e] = du.T @ x
    return dx, dWg, dWu, dWd

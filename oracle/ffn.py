"""Expert FFN oracle -- TEST INFRASTRUCTURE ONLY (numpy, float64).

Section 2.1 of the paper (the compute step between dispatch and combine) leaves the
expert function open; the workloads here use the gated SwiGLU feed-forward of the models the
paper traces (Mixtral, DeepSeek-MoE):

    y = ( silu(x Wg^T) * (x Wu^T) ) Wd^T ,   silu(z) = z / (1 + exp(-z)),   no bias.

Inputs are the very bit patterns the GPU receives (bf16 activations, bf16 or block-scaled
OCP FP8-E4M3 weights); they are decoded to float64 and everything is evaluated in float64
with numpy's matmul.  A row's result depends only on the row and on its expert, never on the
slice it sits in.
"""
from __future__ import annotations

import numpy as np


def decode_bf16(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float64: the pattern is the upper half of a float32."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    with np.errstate(invalid="ignore"):
        return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def decode_e4m3(codes: np.ndarray) -> np.ndarray:
    """OCP 8-bit floating point, E4M3 flavour (1 sign, 4 exponent bits with bias 7, 3 mantissa
    bits, no infinities, S.1111.111 is NaN, exponent field 0 is subnormal) -> float64."""
    c = np.ascontiguousarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = (c & 0x7).astype(np.float64)
    normal = (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64))
    subnormal = (m / 8.0) * 2.0 ** -6
    val = np.where(e == 0, subnormal, normal)
    val = np.where((e == 0xF) & ((c & 0x7) == 0x7), np.nan, val)
    return sign * val


def dequant_block128(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """codes uint8[R][C], scales float32[R/128][C/128] -> float64[R][C] = decode(code) * scale of its block."""
    R, C = codes.shape
    w = decode_e4m3(codes).reshape(R // 128, 128, C // 128, 128)
    return (w * scales.astype(np.float64)[:, None, :, None]).reshape(R, C)


def _silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def expert_ffn_sliced(x_bits: np.ndarray, offsets: np.ndarray, E_loc: int, weights, rows: np.ndarray | None = None,
                      return_hidden: bool = False):
    """x_bits uint16[M][d]; offsets int32[S*E_loc+1] (group g = slice*E_loc + expert);
    weights: object with dtype, w_gate/w_up [E_loc][f][d], w_down [E_loc][d][f] (+ s_* for fp8).
    rows: optional sorted row indices to evaluate (others are skipped).
    Returns y float64[len(rows) or M][d] (and the hidden activations h if asked)."""
    offsets = np.asarray(offsets, dtype=np.int64)
    M_used = int(offsets[-1])
    M, d = x_bits.shape
    G = len(offsets) - 1
    assert G % E_loc == 0 and offsets[0] == 0 and np.all(np.diff(offsets) >= 0) and M_used <= M
    if rows is None:
        rows = np.arange(M_used, dtype=np.int64)
    rows = np.asarray(rows, dtype=np.int64)
    group_of_row = np.searchsorted(offsets, rows, side="right") - 1
    expert_of_row = group_of_row % E_loc
    f = weights.w_gate.shape[1]
    y = np.zeros((len(rows), d), dtype=np.float64)
    h_all = np.zeros((len(rows), f), dtype=np.float64) if return_hidden else None
    for e in range(E_loc):
        sel = np.flatnonzero(expert_of_row == e)
        if sel.size == 0:
            continue
        if weights.dtype == "bf16":
            wg, wu, wd = decode_bf16(weights.w_gate[e]), decode_bf16(weights.w_up[e]), decode_bf16(weights.w_down[e])
        else:
            wg = dequant_block128(weights.w_gate[e], weights.s_gate[e])
            wu = dequant_block128(weights.w_up[e], weights.s_up[e])
            wd = dequant_block128(weights.w_down[e], weights.s_down[e])
        x = decode_bf16(x_bits[rows[sel]])
        g = x @ wg.T
        u = x @ wu.T
        h = _silu(g) * u
        y[sel] = h @ wd.T
        if return_hidden:
            h_all[sel] = h
    return (y, h_all) if return_hidden else y


def expert_ffn_sliced_mapped(x_bits: np.ndarray, offsets: np.ndarray, E_loc: int, weights, row_map: np.ndarray,
                             row_gate: np.ndarray | None = None, rows: np.ndarray | None = None):
    """Dispatch gather and combine scatter around the expert FFN (Section 2.1): schedule row m is row row_map[m] of
    x (arrival order) and of the result, which is multiplied by the router weight row_gate[m].
    Returns (y float64[len(rows) or M_used][d], target rows): y[k] belongs at row target[k] of the output."""
    offsets = np.asarray(offsets, dtype=np.int64)
    M_used = int(offsets[-1])
    row_map = np.asarray(row_map, dtype=np.int64)
    assert len(row_map) >= M_used
    if rows is None:
        rows = np.arange(M_used, dtype=np.int64)
    rows = np.asarray(rows, dtype=np.int64)
    gathered = np.zeros((M_used, x_bits.shape[1]), dtype=np.uint16)
    gathered[rows] = x_bits[row_map[rows]]
    y = expert_ffn_sliced(gathered, offsets, E_loc, weights, rows=rows)
    if row_gate is not None:
        y = y * np.asarray(row_gate, dtype=np.float32).astype(np.float64)[rows, None]
    return y, row_map[rows]

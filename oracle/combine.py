"""Combine oracle -- TEST INFRASTRUCTURE ONLY (numpy, float64).

Section 2.1 of the paper: after the expert computation the results are sent back to the rank that owns the
tokens ("combine"); a token's output is the sum of its experts' results weighted by the router:

    out[t] = sum_j gate[t][j] * y[row_of[t][j]]

The definition written out, in float64, one token and one slot at a time.
"""
from __future__ import annotations

import numpy as np

from .ffn import decode_bf16


def combine_topk_sum(y_bits: np.ndarray, row_of: np.ndarray, gate: np.ndarray | None = None) -> np.ndarray:
    """y_bits uint16 [R][d] (bf16 bit patterns), row_of int [T][topk] (outside [0, R): contributes nothing),
    gate float32 [T][topk] or None (= 1) -> out float64 [T][d]."""
    y = decode_bf16(y_bits)
    R, d = y.shape
    T, topk = row_of.shape
    out = np.zeros((T, d), dtype=np.float64)
    for t in range(T):
        for j in range(topk):
            r = int(row_of[t, j])
            if r < 0 or r >= R:
                continue
            w = 1.0 if gate is None else float(np.float32(gate[t, j]))
            out[t] += w * y[r]
    return out

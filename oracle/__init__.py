"""CPU oracle for the MoE circuit-schedule path -- TEST INFRASTRUCTURE ONLY.

Plain, slow, obviously-correct implementations used by the tests, the smoke check and the
CPU-baseline leg of the benchmark.  Nothing in the GPU package may import this.  The integer
parts live in moe_oracle.c (plain C, compiled with gcc); the expert FFN is numpy float64.
Pinned (tests marked "not gpu") against brute force over all permutations, scipy's assignment
solver, closed forms and the matching counts the paper prints for its Figure 2 example.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile moe_oracle.c with gcc (plain C, OpenMP only for the batched driver)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", _SRC, "-o", _LIB])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        i32p = ctypes.POINTER(ctypes.c_int32)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        u64p = ctypes.POINTER(ctypes.c_uint64)
        ci = ctypes.c_int
        L.oracle_route_histogram.argtypes = [i32p, ci, ci, ci, ci, i32p, i32p]
        L.oracle_route_histogram.restype = ci
        L.oracle_decompose_greedy.argtypes = [i32p, ci, ci, ci, u8p, i32p, i32p]
        L.oracle_decompose_greedy.restype = ci
        L.oracle_decompose_bvn.argtypes = [i32p, ci, ci, ci, u8p, i32p, i32p, i32p, i32p]
        L.oracle_decompose_bvn.restype = ci
        f64p = ctypes.POINTER(ctypes.c_double)
        L.oracle_sinkhorn_bvn.argtypes = [i32p, ci, ci, ci, ci, ctypes.c_double, u8p, f64p, f64p, f64p, f64p]
        L.oracle_sinkhorn_bvn.restype = ci
        L.oracle_decompose_batch.argtypes = [ci, i32p, ci, ci, ci, ci, u8p, i32p, i32p, i32p, i32p, u64p, ci]
        L.oracle_decompose_batch.restype = ci
        L.oracle_schedule_hash.argtypes = [u8p, i32p, ci, ci]
        L.oracle_schedule_hash.restype = ctypes.c_uint64
        L.oracle_slice_table.argtypes = [i32p, ci, ci, ci, ci, ci, i32p, u8p, i32p, ci, ci, i32p, i32p]
        L.oracle_slice_table.restype = ci
        _lib = L
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct)) if a is not None else None


def bvn_bound(n: int) -> int:
    """Largest possible number of BvN matchings of an n x n matrix: (n-1)^2 + 1."""
    return (n - 1) * (n - 1) + 1


# --------------------------------------------------------------------------------------
def route_histogram(ids: np.ndarray, E: int, want_counts: bool = True):
    """ids int32[N][T][topk] -> (traffic int32[N][N], counts int32[N][E] or None)."""
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    N, T, topk = ids.shape
    traffic = np.empty((N, N), dtype=np.int32)
    counts = np.empty((N, E), dtype=np.int32) if want_counts else None
    rc = _load().oracle_route_histogram(_p(ids, ctypes.c_int32), N, T, topk, E,
                                        _p(traffic, ctypes.c_int32), _p(counts, ctypes.c_int32))
    if rc != 0:
        raise ValueError("oracle_route_histogram: bad arguments")
    return traffic, counts


def decompose_greedy(A: np.ndarray, kmax: int, zero_diag: bool = False):
    """One matrix -> (perms uint8[count][n], durations int32[count], residual int32[n][n])."""
    A = np.ascontiguousarray(A, dtype=np.int32)
    n = A.shape[0]
    perms = np.zeros((max(kmax, 1), n), dtype=np.uint8)
    dur = np.zeros(max(kmax, 1), dtype=np.int32)
    res = np.empty((n, n), dtype=np.int32)
    c = _load().oracle_decompose_greedy(_p(A, ctypes.c_int32), n, kmax, int(zero_diag),
                                        _p(perms, ctypes.c_uint8), _p(dur, ctypes.c_int32), _p(res, ctypes.c_int32))
    if c < 0:
        raise ValueError("oracle_decompose_greedy failed: %d" % c)
    return perms[:c].copy(), dur[:c].copy(), res


def decompose_bvn(A: np.ndarray, kmax: int | None = None, zero_diag: bool = False):
    """One matrix -> (perms, lambdas, padded residual, pad_total, padding)."""
    A = np.ascontiguousarray(A, dtype=np.int32)
    n = A.shape[0]
    if kmax is None:
        kmax = bvn_bound(n)
    perms = np.zeros((max(kmax, 1), n), dtype=np.uint8)
    dur = np.zeros(max(kmax, 1), dtype=np.int32)
    res = np.empty((n, n), dtype=np.int32)
    pad = np.empty((n, n), dtype=np.int32)
    tot = ctypes.c_int32(0)
    c = _load().oracle_decompose_bvn(_p(A, ctypes.c_int32), n, kmax, int(zero_diag), _p(perms, ctypes.c_uint8),
                                     _p(dur, ctypes.c_int32), _p(res, ctypes.c_int32), ctypes.byref(tot),
                                     _p(pad, ctypes.c_int32))
    if c < 0:
        raise ValueError("oracle_decompose_bvn failed: %d" % c)
    return perms[:c].copy(), dur[:c].copy(), res, int(tot.value), pad


def sinkhorn_bvn(A: np.ndarray, kmax: int | None = None, zero_diag: bool = False, iters: int = 100, eps: float = 1e-12):
    """One matrix -> (perms, coefficients float64, scaled matrix, residual, deviation of the row sums from 1)."""
    A = np.ascontiguousarray(A, dtype=np.int32)
    n = A.shape[0]
    if kmax is None:
        kmax = n * n
    perms = np.zeros((max(kmax, 1), n), dtype=np.uint8)
    coef = np.zeros(max(kmax, 1), dtype=np.float64)
    scaled = np.empty((n, n), dtype=np.float64)
    res = np.empty((n, n), dtype=np.float64)
    dev = ctypes.c_double(0.0)
    c = _load().oracle_sinkhorn_bvn(_p(A, ctypes.c_int32), n, kmax, int(zero_diag), int(iters), float(eps),
                                    _p(perms, ctypes.c_uint8), _p(coef, ctypes.c_double), _p(scaled, ctypes.c_double),
                                    _p(res, ctypes.c_double), ctypes.byref(dev))
    if c < 0:
        raise ValueError("oracle_sinkhorn_bvn failed: %d" % c)
    return perms[:c].copy(), coef[:c].copy(), scaled, res, float(dev.value)


def decompose_batch(which: str, mats: np.ndarray, kmax: int, zero_diag: bool = False, nthreads: int = 1,
                    want_perms: bool = True, want_residual: bool = True):
    """Batched driver.  Returns dict(perms, durations, counts, residual, pad_total, hashes);
    entries past counts[b] are zero."""
    mats = np.ascontiguousarray(mats, dtype=np.int32)
    B, n, _ = mats.shape
    perms = np.zeros((B, kmax, n), dtype=np.uint8) if want_perms else None
    dur = np.zeros((B, kmax), dtype=np.int32)
    counts = np.zeros(B, dtype=np.int32)
    res = np.zeros((B, n, n), dtype=np.int32) if want_residual else None
    pad_total = np.zeros(B, dtype=np.int32)
    hashes = np.zeros(B, dtype=np.uint64)
    rc = _load().oracle_decompose_batch(0 if which == "greedy" else 1, _p(mats, ctypes.c_int32), B, n, kmax,
                                        int(zero_diag), _p(perms, ctypes.c_uint8), _p(dur, ctypes.c_int32),
                                        _p(counts, ctypes.c_int32), _p(res, ctypes.c_int32),
                                        _p(pad_total, ctypes.c_int32), _p(hashes, ctypes.c_uint64), int(nthreads))
    if rc != 0:
        raise ValueError("oracle_decompose_batch failed")
    return dict(perms=perms, durations=dur, counts=counts, residual=res, pad_total=pad_total, hashes=hashes)


def schedule_hash(perms: np.ndarray, durations: np.ndarray) -> int:
    perms = np.ascontiguousarray(perms, dtype=np.uint8)
    durations = np.ascontiguousarray(durations, dtype=np.int32)
    count = len(durations)
    n = perms.shape[1] if count else 0
    return int(_load().oracle_schedule_hash(_p(perms, ctypes.c_uint8), _p(durations, ctypes.c_int32), count, n))


def slice_table(ids: np.ndarray, E: int, r: int, traffic: np.ndarray, perms: np.ndarray, durations: np.ndarray,
                kmax: int, want_rows: bool = True):
    """-> (offsets int32[(kmax+2)*E_loc+1], row_src int32[M] or None)."""
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    N, T, topk = ids.shape
    traffic = np.ascontiguousarray(traffic, dtype=np.int32)
    count = len(durations)
    pp = np.zeros((max(kmax, 1), N), dtype=np.uint8)
    dd = np.zeros(max(kmax, 1), dtype=np.int32)
    pp[:count] = perms
    dd[:count] = durations
    e_loc = E // N
    offsets = np.zeros((kmax + 2) * e_loc + 1, dtype=np.int32)
    rows = np.full(int(traffic[:, r].sum()), -1, dtype=np.int32) if want_rows else None
    M = _load().oracle_slice_table(_p(ids, ctypes.c_int32), N, T, topk, E, r, _p(traffic, ctypes.c_int32),
                                   _p(pp, ctypes.c_uint8), _p(dd, ctypes.c_int32), count, kmax,
                                   _p(offsets, ctypes.c_int32), _p(rows, ctypes.c_int32))
    if M < 0:
        raise ValueError("oracle_slice_table: bad arguments")
    return offsets, rows


from .ffn import expert_ffn_sliced, expert_ffn_sliced_mapped, decode_bf16, decode_e4m3, dequant_block128  # noqa: E402,F401
from .combine import combine_topk_sum  # noqa: E402,F401
from .ffn_backward import expert_ffn_backward_sliced  # noqa: E402,F401

"""Python binding of libmoecircuit (MI355X / gfx950).

Argument marshalling only: every step of the path runs in the HIP kernels behind the C ABI
declared in include/moe_circuit.h.  torch is used for device memory and streams.  There is no
CPU fallback: if the shared library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import glob
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_HERE, "csrc")
_LIB_PATH = os.path.join(_HERE, "libmoecircuit.so")
_INCLUDE = os.path.join(os.path.dirname(_HERE), "include")

MOE_DECOMP_ZERO_DIAGONAL = 1
MOE_DECOMP_RESIDUAL_I32 = 2
MOE_DECOMP_RESIDUAL_U16 = 4
MOE_W_BF16 = 0
MOE_W_FP8_E4M3_B128 = 1
MOE_MAX_RANKS = 128

_STATUS = {0: "MOE_OK", -1: "MOE_ERR_INVALID_ARG", -2: "MOE_ERR_UNSUPPORTED_SHAPE", -3: "MOE_ERR_WORKSPACE",
           -4: "MOE_ERR_HIP"}

EXPORTS = [
    "moe_route_histogram", "moe_decompose_greedy", "moe_decompose_bvn", "moe_slice_table_workspace_bytes",
    "moe_slice_table", "moe_ffn_workspace_bytes", "moe_ffn_expanded_weights_bytes", "moe_expert_ffn_sliced", "moe_kernel_timing_enable",
    "moe_kernel_timing_read", "moe_kernel_timing_select", "moe_last_hip_error", "moe_makespan_model", "moe_order_matchings", "moe_decompose_sinkhorn_bvn", "moe_slice_table_rows_workspace_bytes",
    "moe_slice_table_rows", "moe_expert_ffn_sliced_mapped", "moe_ffn_tile_override",
    "moe_slice_table_static", "moe_decompose_profile", "moe_combine_topk_sum",
    "moe_ffn_backward_workspace_bytes", "moe_expert_ffn_backward_sliced", "moe_probe_mfma_bf16",
]

_lib = None


class MoeError(RuntimeError):
    pass


class CostModel(ctypes.Structure):
    """struct moe_cost_model of moe_circuit.h."""
    _fields_ = [("bytes_per_row", ctypes.c_double), ("bandwidth", ctypes.c_double), ("reconf_s", ctypes.c_double),
                ("kind", ctypes.c_int), ("fixed_s", ctypes.c_double), ("per_row_s", ctypes.c_double),
                ("table_rows", ctypes.POINTER(ctypes.c_double)), ("table_seconds", ctypes.POINTER(ctypes.c_double)),
                ("table_len", ctypes.c_int)]


def build(verbose: bool = False) -> str:
    """Compile every HIP source for gfx950 into libmoecircuit.so (in-tree)."""
    srcs = sorted(glob.glob(os.path.join(_CSRC, "*.hip")))
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", _INCLUDE, "-o", _LIB_PATH] + srcs
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise MoeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return _LIB_PATH


def load():
    """Load the shared library (built beforehand by build()); fails loudly if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise MoeError("libmoecircuit.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    # torch ships its own HIP runtime (soname libamdhip64.so.7); importing it first makes the
    # library bind to that one instead of bringing a second runtime into the process
    import torch  # noqa: F401
    L = ctypes.CDLL(_LIB_PATH)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    L.moe_route_histogram.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp, vp]
    L.moe_route_histogram.restype = ci
    L.moe_decompose_greedy.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp]
    L.moe_decompose_greedy.restype = ci
    L.moe_decompose_profile.argtypes = [vp, ci]
    L.moe_decompose_profile.restype = ci
    L.moe_decompose_bvn.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp, vp]
    L.moe_decompose_bvn.restype = ci
    L.moe_decompose_sinkhorn_bvn.argtypes = [vp, ci, ci, ci, ci, ci, ctypes.c_double, vp, vp, vp, vp, vp, vp, vp]
    L.moe_decompose_sinkhorn_bvn.restype = ci
    L.moe_slice_table_workspace_bytes.argtypes = [ci, ci, ci]
    L.moe_slice_table_workspace_bytes.restype = sz
    L.moe_slice_table.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp, vp, vp, ci, vp, vp, sz, vp]
    L.moe_slice_table.restype = ci
    L.moe_slice_table_static.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp, vp, vp, ci, vp, vp]
    L.moe_slice_table_static.restype = ci
    L.moe_slice_table_rows_workspace_bytes.argtypes = [ci, ci, ci]
    L.moe_slice_table_rows_workspace_bytes.restype = sz
    L.moe_slice_table_rows.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp, vp, vp, ci, vp, vp, vp, vp, sz, vp]
    L.moe_slice_table_rows.restype = ci
    L.moe_expert_ffn_sliced_mapped.argtypes = [vp, vp, ci, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.moe_expert_ffn_sliced_mapped.restype = ci
    L.moe_ffn_workspace_bytes.argtypes = [ci, ci, ci]
    L.moe_ffn_workspace_bytes.restype = sz
    L.moe_ffn_expanded_weights_bytes.argtypes = [ci, ci, ci]
    L.moe_ffn_expanded_weights_bytes.restype = sz
    L.moe_expert_ffn_sliced.argtypes = [vp, vp, ci, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.moe_expert_ffn_sliced.restype = ci
    L.moe_ffn_backward_workspace_bytes.argtypes = [ci, ci, ci, ci]
    L.moe_ffn_backward_workspace_bytes.restype = sz
    L.moe_expert_ffn_backward_sliced.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.moe_expert_ffn_backward_sliced.restype = ci
    L.moe_combine_topk_sum.argtypes = [vp, vp, vp, ci, ci, ci, ci, vp, vp]
    L.moe_combine_topk_sum.restype = ci
    L.moe_probe_mfma_bf16.argtypes = [ci, ci, ci, vp, vp]
    L.moe_probe_mfma_bf16.restype = ci
    L.moe_ffn_tile_override.argtypes = [ci, ci, ci]
    L.moe_ffn_tile_override.restype = ci
    L.moe_kernel_timing_enable.argtypes = [ci]
    L.moe_kernel_timing_enable.restype = ci
    L.moe_kernel_timing_select.argtypes = [ctypes.c_char_p]
    L.moe_kernel_timing_select.restype = ci
    L.moe_kernel_timing_read.argtypes = [ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_float),
                                         ctypes.POINTER(ctypes.c_int), ci]
    L.moe_kernel_timing_read.restype = ci
    L.moe_last_hip_error.argtypes = []
    L.moe_last_hip_error.restype = ctypes.c_char_p
    L.moe_makespan_model.argtypes = [vp, ci, vp, vp, ci, vp, ctypes.POINTER(CostModel), ctypes.POINTER(ctypes.c_double)]
    L.moe_makespan_model.restype = ci
    L.moe_order_matchings.argtypes = [vp, ci, vp, vp, ci, ctypes.POINTER(CostModel), vp]
    L.moe_order_matchings.restype = ci
    _lib = L
    return L


def _check(rc: int, what: str):
    if rc != 0:
        detail = ""
        if rc == -4:
            detail = ": " + (load().moe_last_hip_error() or b"").decode()
        raise MoeError("%s -> %s%s" % (what, _STATUS.get(rc, str(rc)), detail))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev_check(t, dtype, name):
    import torch
    if t is None:
        return
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype:
        raise MoeError("%s must be a contiguous CUDA tensor of dtype %s" % (name, dtype))


# ---------------------------------------------------------------------------------------------
def moe_route_histogram(ids, E: int, traffic=None, expert_counts=None, want_counts: bool = True):
    """ids int32 [N][T][topk] or [L][N][T][topk] -> (traffic [..][N][N], expert_counts [..][N][E] or None)."""
    import torch
    _dev_check(ids, torch.int32, "ids")
    batched = ids.dim() == 4
    L = ids.shape[0] if batched else 1
    N, T, topk = ids.shape[-3:]
    shp = (L, N) if batched else (N,)
    if traffic is None:
        traffic = torch.empty(shp + (N,), dtype=torch.int32, device=ids.device)
    if expert_counts is None and want_counts:
        expert_counts = torch.empty(shp + (E,), dtype=torch.int32, device=ids.device)
    _dev_check(traffic, torch.int32, "traffic")
    _dev_check(expert_counts, torch.int32, "expert_counts")
    _check(load().moe_route_histogram(_ptr(ids), L, N, T, topk, E, _ptr(traffic), _ptr(expert_counts), _stream()),
           "moe_route_histogram")
    return traffic, expert_counts


def _decomp_buffers(mats, kmax, want_perms, want_residual, want_hashes, out):
    import torch
    B, N, _ = mats.shape
    dev = mats.device
    out = dict(out or {})
    if "perms" not in out:
        out["perms"] = torch.zeros((B, kmax, N), dtype=torch.uint8, device=dev) if want_perms else None
    if "durations" not in out:
        out["durations"] = torch.zeros((B, kmax), dtype=torch.int32, device=dev)
    if "counts" not in out:
        out["counts"] = torch.zeros((B,), dtype=torch.int32, device=dev)
    if "residual" not in out:
        out["residual"] = torch.empty((B, N, N), dtype=torch.int32, device=dev) if want_residual else None
    if "hashes" not in out:
        out["hashes"] = torch.zeros((B,), dtype=torch.int64, device=dev) if want_hashes else None
    return out


def moe_decompose_profile(counters=None):
    """Measurement hook: counters = device int64 tensor [capacity][4] that the following greedy / BvN calls fill per
    matrix with (shader cycles, 100 MHz ticks, search steps, searches); None switches recording off."""
    import torch
    if counters is None:
        _check(load().moe_decompose_profile(None, 0), "moe_decompose_profile")
        return
    _dev_check(counters, torch.int64, "counters")
    _check(load().moe_decompose_profile(_ptr(counters), counters.numel() // 4), "moe_decompose_profile")


def moe_decompose_greedy(mats, kmax: int, zero_diag: bool = False, want_perms=True, want_residual=True,
                         want_hashes=False, out=None, residual_bits: int = 0):
    """mats int32 [B][N][N] -> dict(perms, durations, counts, residual, hashes) of device tensors.
    residual_bits: 0 = the library decides how the residual is held on chip, 32 / 16 pin it (same results)."""
    import torch
    _dev_check(mats, torch.int32, "mats")
    B, N, _ = mats.shape
    o = _decomp_buffers(mats, kmax, want_perms, want_residual, want_hashes, out)
    _check(load().moe_decompose_greedy(_ptr(mats), B, N, kmax,
                                       (MOE_DECOMP_ZERO_DIAGONAL if zero_diag else 0)
                                       | {0: 0, 32: MOE_DECOMP_RESIDUAL_I32, 16: MOE_DECOMP_RESIDUAL_U16}[residual_bits],
                                       _ptr(o["perms"]), _ptr(o["durations"]), _ptr(o["counts"]), _ptr(o["residual"]),
                                       _ptr(o["hashes"]), _stream()), "moe_decompose_greedy")
    return o


def moe_decompose_bvn(mats, kmax: int, zero_diag: bool = False, want_perms=True, want_residual=True,
                      want_hashes=False, out=None):
    """As moe_decompose_greedy, plus pad_total int32 [B]."""
    import torch
    _dev_check(mats, torch.int32, "mats")
    B, N, _ = mats.shape
    o = _decomp_buffers(mats, kmax, want_perms, want_residual, want_hashes, out)
    if "pad_total" not in o:
        o["pad_total"] = torch.zeros((B,), dtype=torch.int32, device=mats.device)
    _check(load().moe_decompose_bvn(_ptr(mats), B, N, kmax, MOE_DECOMP_ZERO_DIAGONAL if zero_diag else 0,
                                    _ptr(o["perms"]), _ptr(o["durations"]), _ptr(o["counts"]), _ptr(o["residual"]),
                                    _ptr(o["pad_total"]), _ptr(o["hashes"]), _stream()), "moe_decompose_bvn")
    return o


def moe_decompose_sinkhorn_bvn(mats, kmax: int, zero_diag: bool = False, sweeps: int = 100, eps: float = 1e-12,
                               want_perms=True, want_scaled=True, want_residual=True):
    """mats int32 [B][N][N] -> dict(perms uint8 [B][kmax][N], coeffs float64 [B][kmax], counts, scaled, residual, deviation)."""
    import torch
    _dev_check(mats, torch.int32, "mats")
    B, N, _ = mats.shape
    dev = mats.device
    o = dict(perms=torch.zeros((B, kmax, N), dtype=torch.uint8, device=dev) if want_perms else None,
             coeffs=torch.zeros((B, kmax), dtype=torch.float64, device=dev),
             counts=torch.zeros((B,), dtype=torch.int32, device=dev),
             scaled=torch.empty((B, N, N), dtype=torch.float64, device=dev) if want_scaled else None,
             residual=torch.empty((B, N, N), dtype=torch.float64, device=dev) if want_residual else None,
             deviation=torch.zeros((B,), dtype=torch.float64, device=dev))
    _check(load().moe_decompose_sinkhorn_bvn(_ptr(mats), B, N, kmax, MOE_DECOMP_ZERO_DIAGONAL if zero_diag else 0,
                                             int(sweeps), float(eps), _ptr(o["perms"]), _ptr(o["coeffs"]), _ptr(o["counts"]),
                                             _ptr(o["scaled"]), _ptr(o["residual"]), _ptr(o["deviation"]), _stream()),
           "moe_decompose_sinkhorn_bvn")
    return o


def moe_slice_table(ids, E: int, r: int, traffic, perms, durations, count, kmax: int, offsets=None, workspace=None):
    """ids [N][T][topk], traffic [N][N], perms uint8 [kmax][N], durations [kmax], count [1] -> offsets."""
    import torch
    _dev_check(ids, torch.int32, "ids")
    _dev_check(traffic, torch.int32, "traffic")
    _dev_check(perms, torch.uint8, "perms")
    _dev_check(durations, torch.int32, "durations")
    _dev_check(count, torch.int32, "count")
    N, T, topk = ids.shape
    e_loc = E // N
    if offsets is None:
        offsets = torch.empty(((kmax + 2) * e_loc + 1,), dtype=torch.int32, device=ids.device)
    need = load().moe_slice_table_workspace_bytes(N, kmax, E)
    if workspace is None:
        workspace = torch.empty((max(need, 1),), dtype=torch.uint8, device=ids.device)
    _check(load().moe_slice_table(_ptr(ids), N, T, topk, E, r, _ptr(traffic), _ptr(perms), _ptr(durations), _ptr(count),
                                  kmax, _ptr(offsets), _ptr(workspace), workspace.numel(), _stream()), "moe_slice_table")
    return offsets


def moe_slice_table_static(ids, E: int, r: int, traffic, perms, durations, count, kmax: int, offsets):
    """moe_slice_table on the library's built-in work area; `offsets` int32 [(kmax+2)*E_loc+1] is the caller's.
    Nothing is allocated here or in the library."""
    N, T, topk = ids.shape
    _check(load().moe_slice_table_static(_ptr(ids), N, T, topk, E, r, _ptr(traffic), _ptr(perms), _ptr(durations), _ptr(count),
                                         kmax, _ptr(offsets), _stream()), "moe_slice_table_static")
    return offsets


def moe_slice_table_rows(ids, E: int, r: int, traffic, perms, durations, count, kmax: int, M: int, offsets=None,
                         want_arrival=True, want_assignment=True, workspace=None):
    """moe_slice_table plus the row map: -> (offsets, row_arrival int32 [M] or None, row_assignment int32 [M] or None);
    M = number of assignments destined to r (column sum of traffic)."""
    import torch
    _dev_check(ids, torch.int32, "ids")
    _dev_check(traffic, torch.int32, "traffic")
    _dev_check(perms, torch.uint8, "perms")
    _dev_check(durations, torch.int32, "durations")
    _dev_check(count, torch.int32, "count")
    N, T, topk = ids.shape
    e_loc = E // N
    if offsets is None:
        offsets = torch.empty(((kmax + 2) * e_loc + 1,), dtype=torch.int32, device=ids.device)
    arr = torch.full((M,), -1, dtype=torch.int32, device=ids.device) if want_arrival else None
    asg = torch.full((M,), -1, dtype=torch.int32, device=ids.device) if want_assignment else None
    need = load().moe_slice_table_rows_workspace_bytes(N, kmax, E)
    if workspace is None:
        workspace = torch.empty((max(need, 1),), dtype=torch.uint8, device=ids.device)
    _check(load().moe_slice_table_rows(_ptr(ids), N, T, topk, E, r, _ptr(traffic), _ptr(perms), _ptr(durations), _ptr(count),
                                       kmax, _ptr(offsets), _ptr(arr), _ptr(asg), _ptr(workspace), workspace.numel(),
                                       _stream()), "moe_slice_table_rows")
    return offsets, arr, asg


def moe_ffn_workspace_bytes(M: int, d: int, f: int) -> int:
    return int(load().moe_ffn_workspace_bytes(M, d, f))


def moe_ffn_expanded_weights_bytes(E_loc: int, d: int, f: int) -> int:
    """Extra workspace that lets a call with fp8 weights and many rows expand them to bf16 once."""
    return int(load().moe_ffn_expanded_weights_bytes(E_loc, d, f))


def moe_expert_ffn_sliced_mapped(x, offsets, S: int, E_loc: int, w_gate, w_up, w_down, row_map, row_gate=None,
                                 s_gate=None, s_up=None, s_down=None, y=None, workspace=None):
    """As moe_expert_ffn_sliced with x and y in arrival order: schedule row m is row row_map[m] of both, and its
    result is scaled by row_gate[m]."""
    import torch
    _dev_check(row_map, torch.int32, "row_map")
    _dev_check(row_gate, torch.float32, "row_gate")
    return moe_expert_ffn_sliced(x, offsets, S, E_loc, w_gate, w_up, w_down, s_gate, s_up, s_down, y, workspace,
                                 _row_map=row_map, _row_gate=row_gate)


def moe_expert_ffn_sliced(x, offsets, S: int, E_loc: int, w_gate, w_up, w_down, s_gate=None, s_up=None, s_down=None,
                          y=None, workspace=None, _row_map=None, _row_gate=None):
    """x bf16 [M][d]; offsets int32 [S*E_loc+1]; bf16 weights (w_gate,w_up [E_loc][f][d], w_down [E_loc][d][f]) or
    uint8 E4M3 codes with float32 block scales -> y bf16 [M][d]."""
    import torch
    _dev_check(x, torch.bfloat16, "x")
    _dev_check(offsets, torch.int32, "offsets")
    M, d = x.shape
    f = w_gate.shape[1]
    fp8 = w_gate.dtype == torch.uint8
    wdt = torch.uint8 if fp8 else torch.bfloat16
    for name, w in (("w_gate", w_gate), ("w_up", w_up), ("w_down", w_down)):
        _dev_check(w, wdt, name)
    for name, sc in (("s_gate", s_gate), ("s_up", s_up), ("s_down", s_down)):
        _dev_check(sc, torch.float32, name)
    if tuple(w_gate.shape) != (E_loc, f, d) or tuple(w_up.shape) != (E_loc, f, d) or tuple(w_down.shape) != (E_loc, d, f):
        raise MoeError("weight shapes must be w_gate/w_up [E_loc][f][d], w_down [E_loc][d][f]")
    if offsets.numel() != S * E_loc + 1:
        raise MoeError("offsets must have S*E_loc+1 entries")
    if y is None:
        y = torch.empty_like(x)
    _dev_check(y, torch.bfloat16, "y")
    need = moe_ffn_workspace_bytes(M, d, f)
    if workspace is None:
        if fp8 and M >= 2048 * E_loc:
            need += moe_ffn_expanded_weights_bytes(E_loc, d, f)
        workspace = torch.empty((max(need, 1),), dtype=torch.uint8, device=x.device)
    if _row_map is not None or _row_gate is not None:
        _check(load().moe_expert_ffn_sliced_mapped(_ptr(x), _ptr(offsets), M, S, E_loc, d, f,
                                                   MOE_W_FP8_E4M3_B128 if fp8 else MOE_W_BF16, _ptr(w_gate), _ptr(w_up),
                                                   _ptr(w_down), _ptr(s_gate), _ptr(s_up), _ptr(s_down), _ptr(_row_map),
                                                   _ptr(_row_gate), _ptr(y), _ptr(workspace), workspace.numel(), _stream()),
               "moe_expert_ffn_sliced_mapped")
        return y
    _check(load().moe_expert_ffn_sliced(_ptr(x), _ptr(offsets), M, S, E_loc, d, f,
                                        MOE_W_FP8_E4M3_B128 if fp8 else MOE_W_BF16, _ptr(w_gate), _ptr(w_up),
                                        _ptr(w_down), _ptr(s_gate), _ptr(s_up), _ptr(s_down), _ptr(y), _ptr(workspace),
                                        workspace.numel(), _stream()), "moe_expert_ffn_sliced")
    return y


def moe_expert_ffn_backward_sliced(x, dy, offsets, S: int, E_loc: int, w_gate, w_up, w_down, workspace=None):
    """x, dy bf16 [M][d]; bf16 weights -> dict(dx [M][d], dw_gate, dw_up [E_loc][f][d], dw_down [E_loc][d][f])."""
    import torch
    for name, t in (("x", x), ("dy", dy), ("w_gate", w_gate), ("w_up", w_up), ("w_down", w_down)):
        _dev_check(t, torch.bfloat16, name)
    _dev_check(offsets, torch.int32, "offsets")
    M, d = x.shape
    f = w_gate.shape[1]
    if tuple(dy.shape) != (M, d) or tuple(w_gate.shape) != (E_loc, f, d) or tuple(w_up.shape) != (E_loc, f, d) or tuple(w_down.shape) != (E_loc, d, f):
        raise MoeError("shapes must be x, dy [M][d]; w_gate, w_up [E_loc][f][d]; w_down [E_loc][d][f]")
    if offsets.numel() != S * E_loc + 1:
        raise MoeError("offsets must have S*E_loc+1 entries")
    out = dict(dx=torch.empty_like(x), dw_gate=torch.empty_like(w_gate), dw_up=torch.empty_like(w_up), dw_down=torch.empty_like(w_down))
    need = int(load().moe_ffn_backward_workspace_bytes(M, E_loc, d, f))
    if workspace is None:
        workspace = torch.empty((max(need, 1),), dtype=torch.uint8, device=x.device)
    _check(load().moe_expert_ffn_backward_sliced(_ptr(x), _ptr(dy), _ptr(offsets), M, S, E_loc, d, f, _ptr(w_gate), _ptr(w_up), _ptr(w_down),
                                                 _ptr(out["dx"]), _ptr(out["dw_gate"]), _ptr(out["dw_up"]), _ptr(out["dw_down"]),
                                                 _ptr(workspace), workspace.numel(), _stream()), "moe_expert_ffn_backward_sliced")
    return out


def moe_combine_topk_sum(y, row_of, gate=None, out=None):
    """y bf16 [R][d], row_of int32 [T][topk], gate float32 [T][topk] or None -> out bf16 [T][d]."""
    import torch
    _dev_check(y, torch.bfloat16, "y")
    _dev_check(row_of, torch.int32, "row_of")
    _dev_check(gate, torch.float32, "gate")
    R, d = y.shape
    T, topk = row_of.shape
    if gate is not None and tuple(gate.shape) != (T, topk):
        raise MoeError("gate must have the shape of row_of")
    if out is None:
        out = torch.empty((T, d), dtype=torch.bfloat16, device=y.device)
    _dev_check(out, torch.bfloat16, "out")
    _check(load().moe_combine_topk_sum(_ptr(y), _ptr(row_of), _ptr(gate), T, topk, d, R, _ptr(out), _stream()),
           "moe_combine_topk_sum")
    return out


def moe_probe_mfma_bf16(data: int, iters: int, workgroups: int, sink=None):
    """Measurement aid: one launch of the register-only MFMA loop (workgroups * 4 * iters * 16 * 32768 flop); returns
    the sink tensor (float32 [workgroups * 256])."""
    import torch
    if sink is None:
        sink = torch.empty((int(workgroups) * 256,), dtype=torch.float32, device="cuda")
    _dev_check(sink, torch.float32, "sink")
    if sink.numel() < int(workgroups) * 256:
        raise MoeError("sink must hold workgroups * 256 floats")
    _check(load().moe_probe_mfma_bf16(int(data), int(iters), int(workgroups), _ptr(sink), _stream()), "moe_probe_mfma_bf16")
    return sink


def moe_ffn_tile_override(tile_rows: int = 0, kernels: int = 0, panel_groups: int = 0):
    """Test / measurement hook: pin the row-block height (64, 128, 256; 0 = automatic), the kernel family (1 = fixed
    shape, 2 = adaptive shape with one launch per phase) and / or the panel width of the tile walk for the following
    FFN calls of this process.  Call with no arguments to restore the defaults."""
    _check(load().moe_ffn_tile_override(int(tile_rows), int(kernels), int(panel_groups)), "moe_ffn_tile_override")


def moe_kernel_timing_enable(on: bool):
    _check(load().moe_kernel_timing_enable(1 if on else 0), "moe_kernel_timing_enable")


def moe_kernel_timing_select(kernel_name=None):
    """Time only the launches of one kernel (None = all)."""
    _check(load().moe_kernel_timing_select(None if kernel_name is None else kernel_name.encode()), "moe_kernel_timing_select")


def moe_kernel_timing_read(cap: int = 32):
    """-> {kernel name: (total_ms, launches)}; synchronises the recorded events and resets the table."""
    names = (ctypes.c_char_p * cap)()
    ms = (ctypes.c_float * cap)()
    n_l = (ctypes.c_int * cap)()
    n = load().moe_kernel_timing_read(names, ms, n_l, cap)
    if n < 0:
        _check(n, "moe_kernel_timing_read")
    return {names[i].decode(): (float(ms[i]), int(n_l[i])) for i in range(n)}


# --------------------------------------------------------------------------------------------- host-side model
def _cost_struct(bytes_per_row, bandwidth, reconf_s, model):
    """model: dict(kind="linear", fixed=..., per_row=...) or dict(kind="table", rows=[...], seconds=[...])."""
    import numpy as np
    c = CostModel()
    c.bytes_per_row, c.bandwidth, c.reconf_s = float(bytes_per_row), float(bandwidth), float(reconf_s)
    keep = []
    if model["kind"] == "linear":
        c.kind, c.fixed_s, c.per_row_s, c.table_len = 0, float(model["fixed"]), float(model["per_row"]), 0
    else:
        xs = np.ascontiguousarray(model["rows"], dtype=np.float64)
        ys = np.ascontiguousarray(model["seconds"], dtype=np.float64)
        keep = [xs, ys]
        c.kind, c.table_len = 1, len(xs)
        c.table_rows = xs.ctypes.data_as(ctypes.POINTER(ctypes.c_double))
        c.table_seconds = ys.ctypes.data_as(ctypes.POINTER(ctypes.c_double))
    return c, keep


def _host_schedule(traffic, perms, durations):
    import numpy as np
    A = np.ascontiguousarray(traffic, dtype=np.int32)
    P = np.ascontiguousarray(perms, dtype=np.uint8).reshape(-1, A.shape[0])
    D = np.ascontiguousarray(durations, dtype=np.int32)
    if P.shape[0] != D.shape[0]:
        raise MoeError("perms and durations disagree on the number of matchings")
    return A, P, D


def moe_makespan_model(traffic, perms, durations, bytes_per_row, bandwidth, reconf_s, model, order=None):
    """Host arrays (numpy) -> dict(sequential, overlap, ideal, comm, compute) in seconds."""
    import numpy as np
    A, P, D = _host_schedule(traffic, perms, durations)
    c, keep = _cost_struct(bytes_per_row, bandwidth, reconf_s, model)
    O = None if order is None else np.ascontiguousarray(order, dtype=np.int32)
    out = (ctypes.c_double * 5)()
    vp = ctypes.c_void_p
    _check(load().moe_makespan_model(vp(A.ctypes.data), A.shape[0], vp(P.ctypes.data), vp(D.ctypes.data), P.shape[0],
                                     None if O is None else vp(O.ctypes.data), ctypes.byref(c), out), "moe_makespan_model")
    del keep
    return dict(zip(("sequential", "overlap", "ideal", "comm", "compute"), [float(v) for v in out]))


def moe_order_matchings(traffic, perms, durations, bytes_per_row, bandwidth, reconf_s, model):
    """Host arrays (numpy) -> int32 [K] play order by Johnson's rule."""
    import numpy as np
    A, P, D = _host_schedule(traffic, perms, durations)
    c, keep = _cost_struct(bytes_per_row, bandwidth, reconf_s, model)
    order = np.zeros((P.shape[0],), dtype=np.int32)
    vp = ctypes.c_void_p
    _check(load().moe_order_matchings(vp(A.ctypes.data), A.shape[0], vp(P.ctypes.data), vp(D.ctypes.data), P.shape[0],
                                      ctypes.byref(c), vp(order.ctypes.data)), "moe_order_matchings")
    del keep
    return order

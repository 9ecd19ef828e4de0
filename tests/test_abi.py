"""The C-ABI library loads and exports every function include/moe_circuit.h declares (no GPU
needed: nothing is computed), and the binding refuses to work without it."""
import ctypes
import os
import re

import pytest

import paper_2605_26845_amd as moe

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "moe_circuit.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    if not os.path.exists(moe._LIB_PATH):
        moe.build()
    lib = ctypes.CDLL(moe._LIB_PATH)
    names = declared_functions()
    assert len(names) >= 10
    for n in names:
        assert hasattr(lib, n), "missing export: " + n
    assert sorted(moe.EXPORTS) == names


def test_host_side_argument_checks_need_no_gpu():
    L = moe.load()
    # sizes and argument errors are decided on the host before anything is enqueued
    assert L.moe_ffn_workspace_bytes(1024, 256, 512) >= 1024 * 512 * 2
    assert L.moe_slice_table_workspace_bytes(8, 4, 8) > 0
    assert L.moe_slice_table_workspace_bytes(8, 4, 9) == 0
    assert L.moe_route_histogram(None, 1, 4, 4, 1, 6, None, None, None) == -1          # traffic missing
    assert L.moe_decompose_greedy(None, 1, 200, 4, 0, None, None, ctypes.c_void_p(8), None, None, None) == -1
    assert L.moe_decompose_greedy(ctypes.c_void_p(8), 1, 200, 4, 0, None, None, ctypes.c_void_p(8), None, None, None) == -2
    # both pins of the residual width at once
    assert L.moe_decompose_greedy(ctypes.c_void_p(8), 1, 4, 1, 2 | 4, None, None, ctypes.c_void_p(8), None, None, None) == -1
    assert L.moe_decompose_profile(None, 3) == -1 and L.moe_decompose_profile(None, 0) == 0
    assert L.moe_ffn_tile_override(100, 0, 0) == -1 and L.moe_ffn_tile_override(0, 3, 0) == -1
    assert L.moe_ffn_tile_override(0, 0, -1) == -1 and L.moe_ffn_tile_override(0, 0, 0) == 0
    # a schedule too long for the built-in work area of the allocation-free slice table
    assert L.moe_slice_table_static(ctypes.c_void_p(8), 8, 4, 1, 8, 0, ctypes.c_void_p(8), ctypes.c_void_p(8), ctypes.c_void_p(8),
                                    ctypes.c_void_p(8), 70000, ctypes.c_void_p(8), None) == -3
    # the FFN takes any number of rows below 2^31, but 32-bit offsets inside one expert's matrices
    assert L.moe_expert_ffn_sliced(ctypes.c_void_p(4096), ctypes.c_void_p(8), 4, 1, 1, 1 << 16, 1 << 15, 0, ctypes.c_void_p(4096),
                                   ctypes.c_void_p(4096), ctypes.c_void_p(4096), None, None, None, ctypes.c_void_p(4096),
                                   None, 0, None) == -2
    assert L.moe_expert_ffn_sliced(ctypes.c_void_p(8), ctypes.c_void_p(8), 4, 1, 1, 100, 128, 0, ctypes.c_void_p(8),
                                   ctypes.c_void_p(8), ctypes.c_void_p(8), None, None, None, ctypes.c_void_p(8),
                                   None, 0, None) == -2                                  # d % 256 != 0
    # operands are moved in 16-byte pieces: a pointer that is only 8-byte aligned is refused, before the workspace check
    ok, odd = ctypes.c_void_p(4096), ctypes.c_void_p(4104)
    for bad in range(5):
        ptrs = [odd if k == bad else ok for k in range(5)]                                # x, w_gate, w_up, w_down, y
        assert L.moe_expert_ffn_sliced(ptrs[0], ctypes.c_void_p(8), 4, 1, 1, 256, 128, 0, ptrs[1], ptrs[2], ptrs[3],
                                       None, None, None, ptrs[4], ok, 1 << 30, None) == -1
    assert L.moe_expert_ffn_sliced(ok, ctypes.c_void_p(8), 4, 1, 1, 256, 128, 0, ok, ok, ok, None, None, None, ok,
                                   None, 0, None) == -3                                  # aligned, workspace missing
    assert L.moe_kernel_timing_read(None, None, None, 0) == 0


def test_probe_argument_checks_need_no_gpu():
    L = moe.load()
    sink = ctypes.c_void_p(4096)
    assert L.moe_probe_mfma_bf16(2, 10, 1, sink, None) == -1          # data is 0 or 1
    assert L.moe_probe_mfma_bf16(1, 0, 1, sink, None) == -1           # at least one iteration
    assert L.moe_probe_mfma_bf16(1, 10, 5000, sink, None) == -1       # at most 4096 workgroups
    assert L.moe_probe_mfma_bf16(1, 10, 1, None, None) == -1          # the sink is required


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(moe, "_lib", None)
    monkeypatch.setattr(moe, "_LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(moe.MoeError):
        moe.load()

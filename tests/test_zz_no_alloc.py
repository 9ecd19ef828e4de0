"""moe_slice_table_static (the entry point that allocates nothing: its work area is a fixed array inside the library's
device image) against moe_slice_table, through the C ABI, on two calls in a row, the second on a smaller input."""
import numpy as np
import pytest
import torch

import oracle
import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def schedule(lib, cfg, which):
    ids = workloads.config_routing(cfg)
    d_ids = dev(ids)
    traffic, _ = lib.moe_route_histogram(d_ids, cfg.E)
    kmax = cfg.kmax if which == "greedy" else oracle.bvn_bound(cfg.N)
    fn = lib.moe_decompose_greedy if which == "greedy" else lib.moe_decompose_bvn
    sched = fn(traffic.unsqueeze(0), kmax, zero_diag=True)
    torch.cuda.synchronize()
    return ids, d_ids, traffic, sched, kmax


def test_slice_table_static_matches_slice_table(lib):
    print("slice table without a caller's workspace: c2 BvN schedule, then the tiny greedy one", flush=True)
    L = lib.load()
    cases = [(workloads.CONFIGS["c2"], "bvn"), (workloads.CONFIGS["tiny"], "greedy")]        # large, then small
    prepared = []
    for cfg, which in cases:
        ids, d_ids, traffic, sched, kmax = schedule(lib, cfg, which)
        r = int(traffic.sum(0).argmax().item())
        want = lib.moe_slice_table(d_ids, cfg.E, r, traffic, sched["perms"][0], sched["durations"][0], sched["counts"], kmax)
        got = torch.full_like(want, -7)                                   # the caller's output buffer, made beforehand
        prepared.append((cfg, which, ids, d_ids, traffic, sched, kmax, r, want, got))
    torch.cuda.synchronize()
    for cfg, which, ids, d_ids, traffic, sched, kmax, r, want, got in prepared:                # back to back, nothing allocated in between
        assert L.moe_slice_table_workspace_bytes(cfg.N, kmax, cfg.E) <= (4 << 20)
        lib.moe_slice_table_static(d_ids, cfg.E, r, traffic, sched["perms"][0], sched["durations"][0], sched["counts"], kmax, got)
    torch.cuda.synchronize()
    for cfg, which, ids, d_ids, traffic, sched, kmax, r, want, got in prepared:
        assert torch.equal(got, want), (cfg.name, which)
        th = traffic.cpu().numpy()
        if which == "greedy":
            rp, rd, _ = oracle.decompose_greedy(th, kmax, zero_diag=True)
        else:
            rp, rd, _, _, _ = oracle.decompose_bvn(th, kmax, zero_diag=True)
        ref, _ = oracle.slice_table(ids, cfg.E, r, th, rp, rd, kmax, want_rows=False)
        assert np.array_equal(got.cpu().numpy(), ref), (cfg.name, which)
    # a schedule whose work area would not fit is refused before anything is enqueued
    big_k = 70000
    assert L.moe_slice_table_workspace_bytes(8, big_k, 8) > (4 << 20)
    with pytest.raises(lib.MoeError, match="MOE_ERR_WORKSPACE"):
        cfg, which, ids, d_ids, traffic, sched, kmax, r, want, got = prepared[1]
        lib.moe_slice_table_static(d_ids, cfg.E, r, traffic, dev(np.zeros((big_k, cfg.N), dtype=np.uint8)),
                                   dev(np.zeros(big_k, dtype=np.int32)), sched["counts"], big_k,
                                   torch.empty(((big_k + 2) * cfg.E_loc + 1,), dtype=torch.int32, device=DEV))

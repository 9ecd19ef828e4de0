"""Pins for the histogram, slice-table and FFN oracles and for the input packers (CPU only)."""
import numpy as np
import pytest
import torch

import oracle
import workloads


# ---------------------------------------------------------------- histogram
@pytest.mark.parametrize("name", ["tiny", "c2"])
def test_histogram_matches_bincount_and_row_sums(name):
    cfg = workloads.CONFIGS[name]
    ids = workloads.config_routing(cfg)
    traffic, counts = oracle.route_histogram(ids, cfg.E)
    N = cfg.N
    for s in range(N):
        assert np.array_equal(counts[s], np.bincount(ids[s].ravel(), minlength=cfg.E))
        assert np.array_equal(traffic[s], np.bincount(ids[s].ravel() // cfg.E_loc, minlength=N))
    assert (traffic.sum(1) == cfg.T * cfg.topk).all()                  # every assignment counted once
    assert np.array_equal(traffic, counts.reshape(N, N, cfg.E_loc).sum(2))
    # invariant under permuting tokens within a rank
    rng = np.random.default_rng(0)
    shuffled = np.stack([ids[s][rng.permutation(cfg.T)] for s in range(N)])
    t2, c2 = oracle.route_histogram(shuffled, cfg.E)
    assert np.array_equal(t2, traffic) and np.array_equal(c2, counts)


def test_histogram_ignores_invalid_ids():
    ids = np.array([[[0, 3], [-1, 2], [4, 1], [7, 7]]], dtype=np.int32).repeat(2, axis=0)   # N=2, E=4
    traffic, counts = oracle.route_histogram(ids, 4)
    assert np.array_equal(counts[0], [1, 1, 1, 1]) and np.array_equal(traffic[0], [2, 2])
    t_only, none = oracle.route_histogram(ids, 4, want_counts=False)
    assert none is None and np.array_equal(t_only, traffic)


# ---------------------------------------------------------------- slice table
def _replay_shipped(traffic, perms, durations, r):
    """tokens delivered to r by each matching, from the rule 'ship min(remaining, duration)'."""
    N = traffic.shape[0]
    rem = traffic[:, r].astype(np.int64).copy()
    rem[r] = 0
    out = []
    for t in range(len(durations)):
        s = int(np.flatnonzero(perms[t] == r)[0])
        ship = 0 if s == r else min(rem[s], int(durations[t]))
        rem[s] -= ship
        out.append((s, ship))
    return out, rem


@pytest.mark.parametrize("name,which", [("tiny", "greedy"), ("tiny", "bvn"), ("c2", "greedy"), ("c2", "bvn")])
def test_slice_table_properties(name, which):
    cfg = workloads.CONFIGS[name]
    ids = workloads.config_routing(cfg)
    N, E_loc = cfg.N, cfg.E_loc
    traffic, counts = oracle.route_histogram(ids, cfg.E)
    r = int(np.argmax(traffic.sum(0)))
    if which == "greedy":
        kmax = cfg.kmax
        perms, dur, _ = oracle.decompose_greedy(traffic, kmax, zero_diag=True)
    else:
        kmax = oracle.bvn_bound(N)
        perms, dur, _, _, _ = oracle.decompose_bvn(traffic, kmax, zero_diag=True)
    offsets, rows = oracle.slice_table(ids, cfg.E, r, traffic, perms, dur, kmax)
    S = kmax + 2
    M = int(traffic[:, r].sum())
    assert offsets[0] == 0 and offsets[-1] == M and (np.diff(offsets) >= 0).all()
    flat = ids.reshape(-1)
    per_src = cfg.T * cfg.topk
    # the rows over all slices are exactly the assignments destined to r, each once
    assert np.array_equal(np.sort(rows), np.flatnonzero(flat // E_loc == r))
    sizes = np.diff(offsets).reshape(S, E_loc)
    shipped, rem = _replay_shipped(traffic, perms, dur, r)
    assert sizes[0].sum() == traffic[r, r]                              # slice 0 = local pairs
    for t, (s, ship) in enumerate(shipped):
        assert sizes[1 + t].sum() == ship                               # slice sizes = shipped amounts
    assert sizes[1 + len(dur):S - 1].sum() == 0                         # unused matching slots stay empty
    assert sizes[S - 1].sum() == rem.sum()                              # the rest
    for sl in range(S):
        for e in range(E_loc):
            g = sl * E_loc + e
            rr = rows[offsets[g]:offsets[g + 1]]
            assert (flat[rr] == r * E_loc + e).all()                    # grouped by local expert
            src = rr // per_src
            if sl == 0:
                assert (src == r).all()
            elif sl < S - 1 and rr.size:
                assert (src == shipped[sl - 1][0]).all()                # one source per matching
            assert (np.diff(src) >= 0).all()
            assert all((np.diff(rr[src == s]) > 0).all() for s in np.unique(src))   # stable
    # first-in-first-out: for a source the slices it feeds are met in schedule order
    slice_of_row = np.repeat(np.arange(S * E_loc) // E_loc, np.diff(offsets))
    for s in range(N):
        mine = np.flatnonzero(rows // per_src == s)
        order = np.argsort(rows[mine])
        assert (np.diff(slice_of_row[mine][order]) >= 0).all()


def test_slice_table_hand_example():
    # N=2 ranks, E=2, one expert per rank, r=1. Source 0 sends 3 assignments to rank 1.
    ids = np.array([[[1], [0], [1], [1]], [[1], [0], [0], [1]]], dtype=np.int32)
    traffic, _ = oracle.route_histogram(ids, 2)
    assert np.array_equal(traffic, [[1, 3], [2, 2]])
    perms = np.array([[1, 0], [1, 0]], dtype=np.uint8)
    dur = np.array([2, 5], dtype=np.int32)          # first matching ships 2 of the 3, second the last one
    offsets, rows = oracle.slice_table(ids, 2, 1, traffic, perms, dur, kmax=3)
    assert list(offsets) == [0, 2, 4, 5, 5, 5]
    assert list(rows) == [4, 7, 0, 2, 3]


# ---------------------------------------------------------------- FFN
def _torch_ffn(x, wg, wu, wd):
    x, wg, wu, wd = (torch.from_numpy(np.ascontiguousarray(a)).double() for a in (x, wg, wu, wd))
    return ((torch.nn.functional.silu(x @ wg.T) * (x @ wu.T)) @ wd.T).numpy()


def test_decoders_match_torch_dtypes():
    bits = np.arange(0, 65536, dtype=np.uint32).astype(np.uint16)
    ref = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).double().numpy()
    got = oracle.decode_bf16(bits)
    ok = ~np.isnan(ref)
    assert np.array_equal(got[ok], ref[ok]) and np.isnan(got[~ok]).all()
    codes = np.arange(256, dtype=np.uint8)
    ref8 = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).double().numpy()
    got8 = oracle.decode_e4m3(codes)
    ok = ~np.isnan(ref8)
    assert np.array_equal(got8[ok], ref8[ok]) and np.isnan(got8[~ok]).all()
    assert got8[0x7E] == 448.0 and got8[0x01] == 2.0 ** -9 and got8[0x38] == 1.0     # format's landmark values


def test_input_packers_match_torch_casts():
    rng = np.random.default_rng(1)
    a = (rng.standard_normal(20000) * np.exp(rng.uniform(-12, 7, 20000))).astype(np.float32)
    a[:8] = [0.0, -0.0, 448.0, 1000.0, -1000.0, 2.0 ** -10, 2.0 ** -9, 465.0]
    t = torch.from_numpy(a)
    assert np.array_equal(workloads.f32_to_bf16_bits(a), t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
    sat = torch.clamp(t, -448.0, 448.0).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(workloads.f32_to_e4m3_bits(a), sat)


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
def test_ffn_matches_torch_float64(dtype):
    E_loc, d, f, M = 2, 256, 384, 200
    W = workloads.ffn_weights(E_loc, d, f, seed=11, dtype=dtype)
    x = workloads.activations(M, d, seed=11)
    offsets = workloads.random_offsets(3 * E_loc, M, seed=2)
    y = oracle.expert_ffn_sliced(x, offsets, E_loc, W)
    xf = torch.from_numpy(x.view(np.int16).copy()).view(torch.bfloat16).double().numpy()
    for g in range(3 * E_loc):
        e = g % E_loc
        if dtype == "bf16":
            dec = lambda b: torch.from_numpy(b.view(np.int16).copy()).view(torch.bfloat16).double().numpy()
            wg, wu, wd = dec(W.w_gate[e]), dec(W.w_up[e]), dec(W.w_down[e])
        else:
            def dec(c, s):
                w = torch.from_numpy(c.copy()).view(torch.float8_e4m3fn).double().numpy()
                return w * np.kron(s.astype(np.float64), np.ones((128, 128)))
            wg, wu, wd = dec(W.w_gate[e], W.s_gate[e]), dec(W.w_up[e], W.s_up[e]), dec(W.w_down[e], W.s_down[e])
        lo, hi = offsets[g], offsets[g + 1]
        ref = _torch_ffn(xf[lo:hi], wg, wu, wd)
        assert np.allclose(y[lo:hi], ref, rtol=1e-12, atol=1e-14)
    assert np.abs(y).max() > 1e-3                                       # not trivially zero


def test_ffn_properties():
    E_loc, d, f, M = 2, 128, 256, 96
    W = workloads.ffn_weights(E_loc, d, f, seed=5)
    x = workloads.activations(M, d, seed=5)
    x[10] = 0                                                           # zero row -> zero output
    off_a = np.array([0, 20, 50, 70, 96], dtype=np.int32)              # 2 slices x 2 experts
    y = oracle.expert_ffn_sliced(x, off_a, E_loc, W)
    assert not y[10].any()
    # a row's result does not depend on the slicing, only on its expert
    off_b = np.array([0, 5, 20, 20, 50, 60, 70, 96, 96], dtype=np.int32)     # same expert per row, 4 slices
    expert_a = (np.searchsorted(off_a, np.arange(M), side="right") - 1) % E_loc
    expert_b = (np.searchsorted(off_b, np.arange(M), side="right") - 1) % E_loc
    same = expert_a == expert_b
    yb = oracle.expert_ffn_sliced(x, off_b, E_loc, W)
    assert same.sum() > 20 and np.allclose(y[same], yb[same], rtol=1e-12, atol=1e-16)   # (BLAS blocking may differ)
    # doubling Wd doubles y exactly (power of two); bf16 exponent bump = +1 in the exponent field
    W2 = workloads.FFNWeights("bf16", W.w_gate, W.w_up, (W.w_down + np.uint16(1 << 7)).astype(np.uint16))
    assert np.array_equal(oracle.expert_ffn_sliced(x, off_a, E_loc, W2), 2.0 * y)
    # sampling rows gives the same rows
    rows = np.array([0, 10, 33, 95])
    assert np.allclose(oracle.expert_ffn_sliced(x, off_a, E_loc, W, rows=rows), y[rows], rtol=1e-12, atol=1e-16)
    # SwiGLU sign structure: swapping gate and up changes the result (catches a transposed operand)
    Wsw = workloads.FFNWeights("bf16", W.w_up, W.w_gate, W.w_down)
    assert not np.allclose(oracle.expert_ffn_sliced(x, off_a, E_loc, Wsw), y)


def test_ffn_mapped_hand_example():
    """Dispatch gather / combine scatter (Section 2.1) on two groups whose source rows, target rows and router weights
    are written out: schedule row m reads arrival row row_map[m], its result times row_gate[m] belongs at the same
    arrival row.  The reference is torch float64 with explicit index_select / index_copy."""
    E_loc, d, f = 2, 128, 256
    W = workloads.ffn_weights(E_loc, d, f, seed=21)
    x = workloads.activations(7, d, seed=22)                            # 7 arrival rows, row 3 is never scheduled
    offsets = np.array([0, 2, 6], dtype=np.int32)                       # group 0 = expert 0: schedule rows 0,1; group 1 = expert 1: rows 2..5
    row_map = np.array([5, 0, 6, 2, 1, 4], dtype=np.int32)
    gate = np.array([0.5, 0.25, 1.0, 0.125, 2.0, 0.75], dtype=np.float32)
    y, target = oracle.expert_ffn_sliced_mapped(x, offsets, E_loc, W, row_map, gate)
    assert list(target) == [5, 0, 6, 2, 1, 4]
    dec = lambda b: torch.from_numpy(np.ascontiguousarray(b).view(np.int16).copy()).view(torch.bfloat16).double()
    xt = dec(x)
    out = torch.full((7, d), float("nan"), dtype=torch.float64)
    for e, (src, gates) in enumerate([([5, 0], [0.5, 0.25]), ([6, 2, 1, 4], [1.0, 0.125, 2.0, 0.75])]):
        idx = torch.tensor(src)
        xe = xt.index_select(0, idx)                                                        # gather
        ye = (torch.nn.functional.silu(xe @ dec(W.w_gate[e]).T) * (xe @ dec(W.w_up[e]).T)) @ dec(W.w_down[e]).T
        out.index_copy_(0, idx, ye * torch.tensor(gates, dtype=torch.float64)[:, None])     # weighted scatter
    got = np.full((7, d), np.nan)
    got[target] = y
    assert np.isnan(got[3]).all() and torch.isnan(out[3]).all()
    keep = [0, 1, 2, 4, 5, 6]
    assert np.allclose(got[keep], out.numpy()[keep], rtol=1e-12, atol=1e-14)
    assert np.abs(got[keep]).max() > 1e-3
    # no gate = unit gate; identity map = the plain call; a row sample returns the same rows and targets
    y1, _ = oracle.expert_ffn_sliced_mapped(x, offsets, E_loc, W, row_map)
    assert np.allclose(y1 * gate.astype(np.float64)[:, None], y, rtol=1e-12, atol=1e-16)
    yi, ti = oracle.expert_ffn_sliced_mapped(x, offsets, E_loc, W, np.arange(6, dtype=np.int32))
    assert list(ti) == list(range(6)) and np.allclose(yi, oracle.expert_ffn_sliced(x, offsets, E_loc, W), rtol=1e-12, atol=1e-16)
    ys, ts = oracle.expert_ffn_sliced_mapped(x, offsets, E_loc, W, row_map, gate, rows=np.array([1, 4]))
    assert list(ts) == [0, 1] and np.allclose(ys, y[[1, 4]], rtol=1e-12, atol=1e-16)
    # the gate belongs to the schedule row, not to the arrival row: permuting the gates changes the result
    yw, _ = oracle.expert_ffn_sliced_mapped(x, offsets, E_loc, W, row_map, gate[row_map.argsort()])
    assert not np.allclose(yw, y)

"""Pins of the makespan oracle (Section 5, Setup) and parity of the library's host-side model with it."""
import itertools

import numpy as np
import pytest

import oracle
from oracle import makespan as om

LIN = dict(kind="linear", fixed=1.0, per_row=0.1)


def test_hand_computed_two_rank_example():
    # one matching that swaps the two ranks; every number below is worked out by hand from the model's rules
    A = [[5, 10], [20, 3]]
    r = om.makespan(A, [[1, 0]], [20], bytes_per_row=1.0, bandwidth=1.0, reconf=0.5, model=LIN)
    # network phase 0.5 + 20 = 20.5; rank 0 receives 20 rows (3.0 s), rank 1 receives 10 (2.0 s); local 1.5 / 1.3
    assert r["sequential"] == pytest.approx(1.5 + 20.5 + 3.0 + 20.5)
    assert r["overlap"] == pytest.approx(20.5 + 3.0 + 20.5)
    assert r["ideal"] == pytest.approx(2 * 20.0 + (1.0 + 0.1 * 25))
    assert r["comm"] == pytest.approx(20.5)
    assert r["compute"] == pytest.approx(1.5 + 3.0)


@pytest.mark.parametrize("n,a", [(4, 7), (8, 100)])
def test_cyclic_shifts_closed_forms(n, a):
    # uniform zero-diagonal traffic, the n-1 cyclic shifts, all durations a: every slice gives every rank a rows
    A = np.full((n, n), a, dtype=np.int64)
    np.fill_diagonal(A, 0)
    perms = [[(i + s) % n for i in range(n)] for s in range(1, n)]
    K = n - 1
    tau = 0.25 + a * 2.0 / 4.0
    # compute much longer than communication: the ranks never wait after the first dispatch
    slow = dict(kind="linear", fixed=0.0, per_row=10.0 * K * tau / a)
    c = 10.0 * K * tau
    r = om.makespan(A, perms, [a] * K, 2.0, 4.0, 0.25, slow)
    assert r["overlap"] == pytest.approx(tau + K * c + tau)
    assert r["sequential"] == pytest.approx(K * (2 * tau + c))
    # free compute: only the network counts, overlap cannot help
    free = dict(kind="linear", fixed=0.0, per_row=0.0)
    r = om.makespan(A, perms, [a] * K, 2.0, 4.0, 0.25, free)
    assert r["overlap"] == pytest.approx(2 * K * tau)
    assert r["sequential"] == pytest.approx(2 * K * tau)
    assert r["ideal"] == pytest.approx(2 * (K * a) * 2.0 / 4.0)


def test_expert_time_table():
    m = dict(kind="table", rows=[64.0, 256.0, 1024.0], seconds=[50e-6, 80e-6, 120e-6])
    assert om.expert_time(0, m) == 0.0
    assert om.expert_time(1, m) == 50e-6                     # floor below the first point
    assert om.expert_time(64, m) == 50e-6
    assert om.expert_time(160, m) == pytest.approx(65e-6)    # midpoint of the first segment
    assert om.expert_time(1024, m) == pytest.approx(120e-6)
    assert om.expert_time(2048, m) == pytest.approx(120e-6 + 1024 * (40e-6 / 768))


def _random_schedule(rng, n, kind):
    A = rng.integers(0, 200, size=(n, n)).astype(np.int32)
    if kind == "greedy":
        perms, dur, res = oracle.decompose_greedy(A, kmax=max(1, n // 2), zero_diag=True)
    else:
        out = oracle.decompose_bvn(A, kmax=oracle.bvn_bound(n), zero_diag=True)
        perms, dur = out[0], out[1]
    return A, perms, dur


@pytest.mark.parametrize("kind", ["greedy", "bvn"])
def test_shipped_amounts_conserve_and_match_slice_sizes(kind):
    rng = np.random.default_rng(5)
    for n in (3, 8, 16):
        A, perms, dur = _random_schedule(rng, n, kind)
        ship, R, local = om.shipped_amounts(A, perms, dur)
        off = A.astype(np.int64).copy()
        np.fill_diagonal(off, 0)
        assert (ship.sum(axis=0) + R.sum(axis=0) == off.sum(axis=0)).all()
        assert (R >= 0).all() and (local == np.diag(A)).all()
        assert (ship.max(axis=1) <= np.asarray(dur)).all()


def test_overlap_never_slower_and_network_is_a_lower_bound():
    rng = np.random.default_rng(11)
    for n in (4, 8):
        for kind in ("greedy", "bvn"):
            A, perms, dur = _random_schedule(rng, n, kind)
            for model in (LIN, dict(kind="table", rows=[8.0, 64.0, 512.0], seconds=[1.0, 1.5, 6.0])):
                r = om.makespan(A, perms, dur, 2.0, 3.0, 0.01, model)
                assert r["overlap"] <= r["sequential"] * (1 + 1e-12)
                assert r["overlap"] >= 2 * r["comm"] * (1 - 1e-12)
                assert r["sequential"] == pytest.approx(2 * r["comm"] + r["compute"])


def _two_stage(a, b, order):
    t1 = t2 = 0.0
    for k in order:
        t1 += a[k]
        t2 = max(t2, t1) + b[k]
    return t2


def test_johnson_order_is_optimal_for_the_two_stage_flow_shop():
    # brute force over all orders; one receiving rank, so dispatch -> compute is exactly a two-machine flow shop
    rng = np.random.default_rng(3)
    for trial in range(30):
        K = int(rng.integers(2, 7))
        n = K + 1
        # matching t sends amount[t] rows from rank t+1 to rank 0 only
        amount = rng.integers(1, 60, size=K)
        A = np.zeros((n, n), dtype=np.int32)
        perms = []
        for t in range(K):
            A[t + 1][0] = amount[t]
            sigma = list(range(n))
            sigma[t + 1], sigma[0] = 0, t + 1
            perms.append(sigma)
        model = dict(kind="linear", fixed=float(rng.uniform(0, 5)), per_row=float(rng.uniform(0.05, 1.0)))
        args = (2.0, float(rng.uniform(1, 8)), float(rng.uniform(0, 2)), model)
        order = om.johnson_order(A, perms, amount, *args)
        a = [args[2] + amount[t] * 2.0 / args[1] for t in range(K)]
        b = [om.expert_time(amount[t], model) for t in range(K)]
        best = min(_two_stage(a, b, p) for p in itertools.permutations(range(K)))
        assert _two_stage(a, b, order) == pytest.approx(best)


# ----------------------------------------------------------------------------------- library (host code) vs oracle
@pytest.mark.parametrize("kind", ["greedy", "bvn"])
def test_library_model_matches_oracle(hostlib, kind):
    import paper_2605_26845_amd as moe
    rng = np.random.default_rng(17)
    models = [LIN, dict(kind="table", rows=[1.0, 64.0, 128.0, 1024.0], seconds=[52e-6, 55e-6, 63e-6, 117e-6])]
    for n in (2, 5, 8, 16):
        A, perms, dur = _random_schedule(rng, n, kind)
        for model in models:
            args = (4096.0, 153e9 if model is not LIN else 7.0, 10e-9, model)
            want = om.makespan(A, perms, dur, *args)
            got = moe.moe_makespan_model(A, perms, dur, *args)
            for k in want:
                assert got[k] == pytest.approx(want[k], rel=1e-12), (n, k)
            order = moe.moe_order_matchings(A, perms, dur, *args)
            assert list(order) == om.johnson_order(A, perms, dur, *args)
            want = om.makespan(A, perms, dur, *args, order=order)
            got = moe.moe_makespan_model(A, perms, dur, *args, order=order)
            for k in want:
                assert got[k] == pytest.approx(want[k], rel=1e-12), (n, k, "ordered")


def test_library_model_argument_errors(hostlib):
    import paper_2605_26845_amd as moe
    A = np.array([[0, 3], [4, 0]], dtype=np.int32)
    with pytest.raises(moe.MoeError):
        moe.moe_makespan_model(A, [[1, 0]], [4], 2.0, 0.0, 0.0, LIN)                       # zero bandwidth
    with pytest.raises(moe.MoeError):
        moe.moe_makespan_model(A, [[1, 0]], [4], 2.0, 1.0, 0.0, LIN, order=[1])           # not a permutation of 0..K-1
    with pytest.raises(moe.MoeError):
        moe.moe_makespan_model(A, [[1, 0]], [4], 2.0, 1.0, 0.0, dict(kind="table", rows=[2.0, 1.0], seconds=[1.0, 1.0]))

"""Pins of the Sinkhorn-Knopp + floating-point BvN oracle (Section 3.1)."""
import itertools

import numpy as np
import pytest

import oracle
import workloads


def dense_matrix(rng, n, lo=1, hi=500):
    return rng.integers(lo, hi, size=(n, n)).astype(np.int32)


def test_scaling_is_a_diagonal_scaling_with_unit_line_sums():
    rng = np.random.default_rng(1)
    for n in (3, 8, 16):
        A = dense_matrix(rng, n)
        _, _, X, _, dev = oracle.sinkhorn_bvn(A, kmax=0, iters=200)
        assert dev < 1e-12
        assert np.allclose(X.sum(axis=0), 1.0, atol=1e-14) and np.allclose(X.sum(axis=1), 1.0, atol=1e-12)
        # X = D1 A D2: cross ratios of 2x2 minors are those of A
        Af = A.astype(np.float64)
        for (i, k, j, l) in [(0, 1, 0, 1), (0, n - 1, 1, n - 1), (1, 2, 0, 2)]:
            assert X[i, j] * X[k, l] / (X[i, l] * X[k, j]) == pytest.approx(Af[i, j] * Af[k, l] / (Af[i, l] * Af[k, j]), rel=1e-12)


def test_closed_forms():
    n = 6
    pi = [3, 0, 5, 1, 2, 4]
    A = np.zeros((n, n), dtype=np.int32)
    for i, j in enumerate(pi):
        A[i, j] = 37
    perms, coef, X, res, dev = oracle.sinkhorn_bvn(A, iters=5)
    assert len(perms) == 1 and list(perms[0]) == pi and coef[0] == 1.0 and dev == 0.0 and not res.any()
    ones = np.ones((n, n), dtype=np.int32)
    perms, coef, X, res, dev = oracle.sinkhorn_bvn(ones, iters=5)
    assert len(perms) == n and list(perms[0]) == list(range(n))
    assert np.allclose(coef, 1.0 / n, rtol=1e-14) and coef.sum() == pytest.approx(1.0, abs=1e-14)
    # already balanced (a sum of permutation matrices with integer weights): scaling only divides by the line sum
    B = 3 * np.eye(n, dtype=np.int32) + 2 * np.roll(np.eye(n, dtype=np.int32), 1, axis=1)
    perms, coef, X, res, dev = oracle.sinkhorn_bvn(B, iters=3)
    assert len(perms) == 2 and sorted(np.round(coef, 12)) == [0.4, 0.6]
    z = np.zeros((4, 4), dtype=np.int32)
    perms, coef, X, res, dev = oracle.sinkhorn_bvn(z, iters=3)
    assert len(perms) == 0


def test_reconstruction_and_counts():
    rng = np.random.default_rng(2)
    for n in (4, 8, 16):
        A = dense_matrix(rng, n)
        perms, coef, X, res, dev = oracle.sinkhorn_bvn(A, iters=300, eps=1e-12)
        acc = res.copy()
        for sigma, lam in zip(perms, coef):
            assert sorted(sigma) == list(range(n)) and lam > 1e-12
            acc[np.arange(n), sigma] += lam
        assert np.allclose(acc, X, atol=1e-13)
        assert coef.sum() == pytest.approx(1.0, abs=1e-9)
        assert res.max() <= 1e-9
        assert len(perms) <= oracle.bvn_bound(n)          # (n-1)^2 + 1; 50 for the paper's 8 x 8 example (Section 5, Results)
    # a dense positive 8 x 8 matrix typically needs close to all of its 50
    A = dense_matrix(np.random.default_rng(9), 8)
    perms, coef, *_ = oracle.sinkhorn_bvn(A, iters=300)
    assert 40 <= len(perms) <= 50


def test_each_step_is_the_lexicographically_first_permutation_in_the_support():
    rng = np.random.default_rng(3)
    for n in (3, 4, 5):
        A = rng.integers(0, 9, size=(n, n)).astype(np.int32) * (rng.random((n, n)) < 0.8)
        A = A.astype(np.int32) + np.eye(n, dtype=np.int32)          # keeps a perfect matching in the support
        eps = 1e-12
        perms, coef, X, res, dev = oracle.sinkhorn_bvn(A, iters=50, eps=eps)
        R = X.copy()
        for sigma, lam in zip(perms, coef):
            first = next(p for p in itertools.permutations(range(n)) if all(R[i, p[i]] > eps for i in range(n)))
            assert list(sigma) == list(first)
            assert lam == min(R[i, sigma[i]] for i in range(n))
            for i in range(n):
                R[i, sigma[i]] -= lam
        # it stopped because nothing decomposable is left (or the cap, not set here)
        assert not any(all(R[i, p[i]] > eps for i in range(n)) for p in itertools.permutations(range(n)))


def test_zero_diagonal_sparse_input_stops_gracefully():
    cfg = workloads.CONFIGS["tiny"]
    ids = workloads.config_routing(cfg)
    traffic, _ = oracle.route_histogram(ids, cfg.E)
    perms, coef, X, res, dev = oracle.sinkhorn_bvn(traffic, zero_diag=True, iters=500)
    assert np.all(np.diag(X) == 0.0) and len(perms) >= cfg.N - 1
    assert coef.sum() <= 1.0 + 1e-9

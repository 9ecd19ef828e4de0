"""Pins for the decomposition oracle (CPU only).  None of these re-type the oracle's own
algorithm: they use brute force over all permutations, scipy's assignment solver, closed forms,
conservation laws and the counts the paper prints for Figure 2."""
import itertools
import os

import numpy as np
import pytest
from scipy.optimize import linear_sum_assignment
from scipy.sparse import csr_matrix
from scipy.sparse.csgraph import maximum_bipartite_matching

import oracle
import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def golden_counts():
    vals = {}
    with open(os.path.join(GOLDEN, "fig2_matching_counts.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            k, v = line.split()
            vals[k] = int(v)
    return vals


# ---------------------------------------------------------------- brute force references
def brute_greedy(A, kmax):
    """Greedy max-weight decomposition by enumerating all n! permutations in lexicographic
    order and replacing the incumbent only on strictly larger weight (Section 3.2; whole
    entries are removed; duration = heaviest pair, Section 3.3)."""
    R = A.astype(np.int64).copy()
    n = R.shape[0]
    out = []
    while len(out) < kmax and R.any():
        best, best_w = None, -1
        for perm in itertools.permutations(range(n)):
            w = sum(R[i, perm[i]] for i in range(n))
            if w > best_w:
                best, best_w = perm, w
        d = max(R[i, best[i]] for i in range(n))
        for i in range(n):
            R[i, best[i]] = 0
        out.append((best, int(d)))
    return out, R


def brute_bvn(Apad, kmax):
    """BvN on an already balanced matrix: first permutation in lexicographic order whose
    entries are all positive, coefficient = smallest of them (Section 3.1)."""
    R = Apad.astype(np.int64).copy()
    n = R.shape[0]
    out = []
    while len(out) < kmax and R.any():
        pick = None
        for perm in itertools.permutations(range(n)):
            if all(R[i, perm[i]] > 0 for i in range(n)):
                pick = perm
                break
        assert pick is not None, "balanced matrix must contain a perfect matching"
        lam = min(R[i, pick[i]] for i in range(n))
        for i in range(n):
            R[i, pick[i]] -= lam
        out.append((pick, int(lam)))
    return out, R


def perm_matrix(perm, n):
    P = np.zeros((n, n), dtype=np.int64)
    P[np.arange(n), np.asarray(perm, dtype=np.int64)] = 1
    return P


# ---------------------------------------------------------------- greedy
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6])
@pytest.mark.parametrize("high", [2, 4, 50])
def test_greedy_equals_brute_force(n, high):
    mats = workloads.random_matrices(12 if n < 6 else 5, n, seed=100 * n + high, density=0.8, high=high)
    for A in mats:
        for kmax in (1, 3, n * n + 1):
            perms, dur, res = oracle.decompose_greedy(A, kmax)
            ref, Rref = brute_greedy(A, kmax)
            assert len(dur) == len(ref)
            for t, (p, d) in enumerate(ref):
                assert tuple(perms[t]) == p, (A, t)
                assert dur[t] == d
            assert np.array_equal(res, Rref)


@pytest.mark.parametrize("n,density,high", [(8, 1.0, 1000), (16, 0.5, 30), (32, 0.3, 5), (64, 1.0, 100000), (128, 0.6, 40000)])
def test_greedy_weight_matches_scipy_and_invariants(n, density, high):
    mats = workloads.random_matrices(3, n, seed=7 + n, density=density, high=high, zero_diag=True)
    for A in mats:
        kmax = 4 * n
        perms, dur, res = oracle.decompose_greedy(A, kmax)
        R = A.astype(np.int64).copy()
        prev_w = None
        shipped = np.zeros_like(R)
        for t in range(len(dur)):
            sig = perms[t].astype(np.int64)
            assert sorted(sig) == list(range(n))                       # a permutation
            rows, cols = linear_sum_assignment(R, maximize=True)       # library optimum (weight only)
            w = R[np.arange(n), sig].sum()
            assert w == R[rows, cols].sum()
            if prev_w is None:
                assert w * n >= A.sum()                                # n cyclic shifts partition A
            else:
                assert w <= prev_w                                     # weights never increase
            prev_w = w
            assert dur[t] == R[np.arange(n), sig].max()
            shipped[np.arange(n), sig] += R[np.arange(n), sig]
            R[np.arange(n), sig] = 0
        assert np.array_equal(R, res)
        assert not res.any()                                           # uncapped: everything shipped
        assert np.array_equal(shipped + res, A)                        # conservation
        nnz = int((A > 0).sum())
        max_line = max((A > 0).sum(0).max(), (A > 0).sum(1).max())
        assert max_line <= len(dur) <= nnz


def test_greedy_lex_rule_on_ties():
    # all-ones: every permutation is optimal; the lexicographically smallest is the identity,
    # then the smallest permutation avoiding the removed entries, and so on: n matchings of weight n
    n = 5
    perms, dur, res = oracle.decompose_greedy(np.ones((n, n), dtype=np.int32), 100)
    assert len(dur) == n and list(perms[0]) == list(range(n)) and all(d == 1 for d in dur)
    assert not res.any()
    # two optima of equal weight: [[1,1],[1,1]] variants
    A = np.array([[3, 3, 0], [3, 3, 0], [0, 0, 1]], dtype=np.int32)
    perms, dur, _ = oracle.decompose_greedy(A, 10)
    assert list(perms[0]) == [0, 1, 2] and list(perms[1]) == [1, 0, 2]


def test_greedy_closed_forms():
    n = 7
    rng = np.random.default_rng(5)
    pi = rng.permutation(n)
    A = (perm_matrix(pi, n) * 9).astype(np.int32)
    perms, dur, res = oracle.decompose_greedy(A, 10)                   # c * P -> one matching (pi, c)
    assert len(dur) == 1 and list(perms[0]) == list(pi) and dur[0] == 9 and not res.any()
    a = np.arange(1, n + 1)
    b = np.arange(2, n + 2)
    perms, dur, _ = oracle.decompose_greedy(np.outer(a, b).astype(np.int32), 1)
    assert list(perms[0]) == list(range(n))                            # rearrangement inequality, unique
    perms, dur, res = oracle.decompose_greedy(np.zeros((n, n), dtype=np.int32), 5)
    assert len(dur) == 0 and not res.any()
    perms, dur, res = oracle.decompose_greedy(np.ones((n, n), dtype=np.int32), 0)     # kmax = 0
    assert len(dur) == 0 and res.sum() == n * n


def test_greedy_cap_returns_residual():
    A = workloads.random_matrices(1, 16, seed=3, zero_diag=True)[0]
    full_p, full_d, _ = oracle.decompose_greedy(A, 1000)
    perms, dur, res = oracle.decompose_greedy(A, 4)
    assert len(dur) == 4 and np.array_equal(perms, full_p[:4]) and np.array_equal(dur, full_d[:4])
    R = A.astype(np.int64).copy()
    for t in range(4):
        R[np.arange(16), perms[t]] = 0
    assert np.array_equal(R, res) and res.any()


def test_greedy_zero_diag_flag_equals_zeroed_input():
    A = workloads.random_matrices(1, 12, seed=9)[0]
    Z = A.copy()
    np.fill_diagonal(Z, 0)
    a = oracle.decompose_greedy(A, 50, zero_diag=True)
    b = oracle.decompose_greedy(Z, 50)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))


def test_paper_figure2_counts():
    """Figure 2: 7 max-weight matchings and 50 BvN matchings for an 8x8 matrix."""
    g = golden_counts()
    n = g["n"]
    cfg = workloads.CONFIGS["tiny"]
    mw_counts, bvn_counts = [], []
    for seed in range(8):
        ids = workloads.route_topk(n, 4096, n, 2, cfg.zipf_s, seed=cfg.seed + seed)
        traffic, _ = oracle.route_histogram(ids, n)
        assert (traffic > 0).all()                                     # dense 8x8
        mw_counts.append(len(oracle.decompose_greedy(traffic, 1000, zero_diag=True)[1]))
        bvn_counts.append(len(oracle.decompose_bvn(traffic)[1]))
    assert max(bvn_counts) == g["bvn_matchings"] == oracle.bvn_bound(n)       # "up to 50"
    assert min(bvn_counts) >= g["bvn_matchings"] - 2
    assert np.median(mw_counts) == g["mw_matchings"]
    assert min(mw_counts) >= g["mw_matchings"]                         # n-1 lines of positive entries


# ---------------------------------------------------------------- BvN
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6])
@pytest.mark.parametrize("high", [3, 40])
def test_bvn_equals_brute_force(n, high):
    mats = workloads.random_matrices(10 if n < 6 else 4, n, seed=55 * n + high, density=0.7, high=high)
    for A in mats:
        for kmax in (2, oracle.bvn_bound(n)):
            perms, lam, res, tot, pad = oracle.decompose_bvn(A, kmax)
            ref, Rref = brute_bvn(A.astype(np.int64) + pad, kmax)
            assert len(lam) == len(ref)
            for t, (p, l) in enumerate(ref):
                assert tuple(perms[t]) == p and lam[t] == l
            assert np.array_equal(res, Rref)


@pytest.mark.parametrize("n,density,high,zd", [(8, 1.0, 1000, False), (16, 0.4, 50, True), (32, 0.2, 7, True), (64, 1.0, 5000, True)])
def test_bvn_invariants(n, density, high, zd):
    mats = workloads.random_matrices(2, n, seed=31 + n, density=density, high=high)
    for A in mats:
        perms, lam, res, tot, pad = oracle.decompose_bvn(A, None, zero_diag=zd)
        A0 = A.astype(np.int64).copy()
        if zd:
            np.fill_diagonal(A0, 0)
        # padding: non-negative, at most 2n-1 entries, equalises all line sums at the largest one
        assert (pad >= 0).all() and (pad > 0).sum() <= 2 * n - 1
        target = max(A0.sum(0).max(), A0.sum(1).max())
        assert tot == target                                            # ideal all-to-all time in tokens
        P = A0 + pad
        assert (P.sum(0) == target).all() and (P.sum(1) == target).all()
        # replay
        R = P.copy()
        for t in range(len(lam)):
            sig = perms[t].astype(np.int64)
            assert sorted(sig) == list(range(n))
            assert lam[t] >= 1 and lam[t] == R[np.arange(n), sig].min()
            R[np.arange(n), sig] -= lam[t]
            assert (R >= 0).all()
            assert (R.sum(0) == R.sum(0)[0]).all() and (R.sum(1) == R.sum(0)[0]).all()
            # a perfect matching must exist in what remains (library routine)
            if R.any() and t % 17 == 0:
                m = maximum_bipartite_matching(csr_matrix((R > 0).astype(np.int8)), perm_type="column")
                assert (m >= 0).all()
        assert not R.any() and not res.any()
        assert lam.sum() == target                                      # sum of coefficients = T*
        assert len(lam) <= (P > 0).sum() - 2 * n + 2 <= oracle.bvn_bound(n)


def test_bvn_closed_forms():
    n = 6
    pi = np.random.default_rng(2).permutation(n)
    perms, lam, res, tot, pad = oracle.decompose_bvn((perm_matrix(pi, n) * 4).astype(np.int32))
    assert len(lam) == 1 and list(perms[0]) == list(pi) and lam[0] == 4 and tot == 4 and not pad.any()
    perms, lam, res, tot, pad = oracle.decompose_bvn(np.ones((n, n), dtype=np.int32))
    assert len(lam) == n and (lam == 1).all() and list(perms[0]) == list(range(n)) and not pad.any()
    perms, lam, res, tot, pad = oracle.decompose_bvn(np.zeros((n, n), dtype=np.int32))
    assert len(lam) == 0 and tot == 0
    # capped: residual is what is left of the padded matrix
    A = workloads.random_matrices(1, 8, seed=77)[0]
    perms, lam, res, tot, pad = oracle.decompose_bvn(A, 5)
    R = A.astype(np.int64) + pad
    for t in range(5):
        R[np.arange(8), perms[t]] -= lam[t]
    assert len(lam) == 5 and np.array_equal(R, res)


def test_bvn_padding_is_the_north_west_corner_fill():
    """Where the padding goes (Section 3.1 needs equal line sums; any non-negative matrix with the right marginals would
    balance, the decomposition differs).  Worked by hand: deficits r_i = T* - row sum, c_j = T* - column sum; start at
    the north-west corner, put min(r_i, c_j) at (i, j), move down when the row is satisfied, right when the column is."""
    # row sums 4,2,1; column sums 5,1,1; T* = 5; r = (1,3,4), c = (0,4,4)
    A = np.array([[4, 0, 0], [1, 1, 0], [0, 0, 1]], dtype=np.int32)
    _, lam, _, tot, pad = oracle.decompose_bvn(A)
    assert tot == 5 and pad.tolist() == [[0, 1, 0], [0, 3, 0], [0, 0, 4]] and lam.sum() == 5
    # row and column deficits tie at every step: r = c = (0,3,2) -> the fill runs down the diagonal
    A = np.array([[5, 1, 0], [0, 2, 1], [1, 0, 3]], dtype=np.int32)
    _, _, _, tot, pad = oracle.decompose_bvn(A)
    assert tot == 6 and pad.tolist() == [[0, 0, 0], [0, 3, 0], [0, 0, 2]]
    # 4 x 4, zero diagonal: row sums 4,3,5,3, column sums 3,4,3,5, T* = 5, r = (1,2,0,2), c = (2,1,2,0);
    # the padding lands on the diagonal too (an idle circuit)
    A = np.array([[0, 3, 1, 0], [2, 0, 0, 1], [0, 1, 0, 4], [1, 0, 2, 0]], dtype=np.int32)
    for zd in (False, True):
        _, _, _, tot, pad = oracle.decompose_bvn(A, zero_diag=zd)
        assert tot == 5 and pad.tolist() == [[1, 0, 0, 0], [1, 1, 0, 0], [0, 0, 0, 0], [0, 0, 2, 0]]
    # the flag zeroes the diagonal before the deficits are taken: 9 on the diagonal would otherwise set T* = 12
    B = A.copy()
    B[2, 2] = 7
    _, _, _, tot, pad = oracle.decompose_bvn(B, zero_diag=True)
    assert tot == 5 and pad.tolist() == [[1, 0, 0, 0], [1, 1, 0, 0], [0, 0, 0, 0], [0, 0, 2, 0]]
    _, _, _, tot, pad = oracle.decompose_bvn(B, zero_diag=False)
    # row sums 4,3,12,3, column sums 3,4,10,5: T* = 12, r = (8,9,0,9), c = (9,8,2,7)
    assert tot == 12 and pad.tolist() == [[8, 0, 0, 0], [1, 8, 0, 0], [0, 0, 0, 0], [0, 0, 2, 7]]
    # and the first matching on a hand-made padded matrix: the lexicographically first permutation inside the support
    A = np.array([[4, 0, 0], [1, 1, 0], [0, 0, 1]], dtype=np.int32)          # padded: [[4,1,0],[1,4,0],[0,0,5]]
    perms, lam, res, _, _ = oracle.decompose_bvn(A)
    assert perms.tolist() == [[0, 1, 2], [1, 0, 2]] and lam.tolist() == [4, 1] and not res.any()


def test_batch_driver_and_hash():
    mats = workloads.random_matrices(6, 16, seed=4, density=0.6, high=20, zero_diag=True)
    for which in ("greedy", "bvn"):
        kmax = 8 if which == "greedy" else oracle.bvn_bound(16)
        out = oracle.decompose_batch(which, mats, kmax, nthreads=3)
        for b, A in enumerate(mats):
            if which == "greedy":
                p, d, r = oracle.decompose_greedy(A, kmax)
            else:
                p, d, r, tot, _ = oracle.decompose_bvn(A, kmax)
                assert out["pad_total"][b] == tot
            c = out["counts"][b]
            assert c == len(d)
            assert np.array_equal(out["perms"][b, :c], p) and np.array_equal(out["durations"][b, :c], d)
            assert np.array_equal(out["residual"][b], r)
            # FNV-1a 64 written out here independently
            h = 14695981039346656037
            for t in range(c):
                for byte in list(p[t]) + list(int(d[t]).to_bytes(4, "little")):
                    h = ((h ^ int(byte)) * 1099511628211) % (1 << 64)
            assert int(out["hashes"][b]) == h == oracle.schedule_hash(p, d)
    # the published FNV-1a test vector: empty input hashes to the offset basis
    assert oracle.schedule_hash(np.zeros((0, 4), np.uint8), np.zeros(0, np.int32)) == 0xCBF29CE484222325

"""GPU parity tests: every call goes through the C ABI (ctypes binding) and is compared with the
CPU oracle on the same seeded inputs -- bit-exact for histogram, decompositions and slice table,
max relative error <= 2e-2 (bf16 weights) / 6e-2 (fp8 weights) for the FFN."""

import numpy as np
import pytest
import torch

import oracle
import workloads

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
FFN_TOL = {"bf16": 2e-2, "fp8": 6e-2}        # the contract: max relative error per (slice, expert) group
# Regression guard beside the contract.  One rounding of h and one of y to bf16 (2^-9 relative each, on sums whose
# terms partly cancel) put the error of these kernels at 3e-3 .. 5e-3 of a group's largest output; a result that is
# still inside the contract but several times that is a defect (a dropped K step, a misplaced scale), not rounding.
FFN_GUARD = {"bf16": 1e-2, "fp8": 1.5e-2}


def check_ffn_error(err, dtype, what=""):
    say("   %s max relative error %.3g" % (what, err))
    assert err <= FFN_TOL[dtype], (what, err)
    assert err <= FFN_GUARD[dtype], ("inside the contract but far above what these kernels have measured", what, err)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def dev_bf16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(DEV).view(torch.bfloat16)


def host_bf16_bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def say(*a):
    print(*a, flush=True)


# ------------------------------------------------------------------------------ histogram
@pytest.mark.parametrize("name", ["tiny", "c2", "c3"])
def test_histogram_configs(lib, name):
    cfg = workloads.CONFIGS[name]
    say("histogram", name)
    ids = workloads.config_routing(cfg)
    traffic, counts = lib.moe_route_histogram(dev(ids), cfg.E)
    torch.cuda.synchronize()
    rt, rc = oracle.route_histogram(ids, cfg.E)
    assert np.array_equal(traffic.cpu().numpy(), rt)
    assert np.array_equal(counts.cpu().numpy(), rc)


@pytest.mark.parametrize("N,T,topk,E,L", [(3, 7, 3, 6, 1), (4, 1, 1, 4, 2), (8, 5000, 5, 64, 3), (2, 40001, 1, 4096, 1),
                                          (16, 0, 2, 16, 1), (5, 33, 2, 640, 4)])
def test_histogram_shapes_and_invalid_ids(lib, N, T, topk, E, L):
    say("histogram shapes", N, T, topk, E, L)
    rng = np.random.default_rng(N * 1000 + T)
    ids = rng.integers(-2, E + 2, size=(L, N, T, topk), dtype=np.int64).astype(np.int32)   # includes invalid ids
    traffic, counts = lib.moe_route_histogram(dev(ids), E)
    t_only, none = lib.moe_route_histogram(dev(ids), E, want_counts=False)
    torch.cuda.synchronize()
    assert none is None
    for l in range(L):
        rt, rc = oracle.route_histogram(ids[l], E)
        assert np.array_equal(traffic[l].cpu().numpy(), rt)
        assert np.array_equal(counts[l].cpu().numpy(), rc)
        assert np.array_equal(t_only[l].cpu().numpy(), rt)


def test_histogram_argument_errors(lib):
    ids = torch.zeros((2, 4, 1), dtype=torch.int32, device=DEV)
    with pytest.raises(lib.MoeError):
        lib.moe_route_histogram(ids, 3)                     # E % N != 0
    with pytest.raises(lib.MoeError):
        lib.moe_route_histogram(ids, 8192)                  # E too large


# ------------------------------------------------------------------------------ decompositions
def check_decomposition(lib, which, mats, kmax, zero_diag):
    B, N, _ = mats.shape
    fn = lib.moe_decompose_greedy if which == "greedy" else lib.moe_decompose_bvn
    sentinel_p, sentinel_d = 0xEE, -777
    out0 = {"perms": torch.full((B, kmax, N), sentinel_p, dtype=torch.uint8, device=DEV),
            "durations": torch.full((B, kmax), sentinel_d, dtype=torch.int32, device=DEV)}
    out = fn(dev(mats), kmax, zero_diag=zero_diag, want_hashes=True, out=out0)
    torch.cuda.synchronize()
    ref = oracle.decompose_batch(which, mats, kmax, zero_diag=zero_diag, nthreads=8)
    counts = out["counts"].cpu().numpy()
    assert np.array_equal(counts, ref["counts"]), (which, N, counts, ref["counts"])
    perms = out["perms"].cpu().numpy()
    dur = out["durations"].cpu().numpy()
    for b in range(B):
        c = counts[b]
        assert np.array_equal(perms[b, :c], ref["perms"][b, :c]), (which, N, b)
        assert np.array_equal(dur[b, :c], ref["durations"][b, :c]), (which, N, b)
        assert (perms[b, c:] == sentinel_p).all() and (dur[b, c:] == sentinel_d).all()    # untouched past count
    assert np.array_equal(out["residual"].cpu().numpy(), ref["residual"])
    assert np.array_equal(out["hashes"].cpu().numpy().view(np.uint64), ref["hashes"])
    if which == "bvn":
        assert np.array_equal(out["pad_total"].cpu().numpy(), ref["pad_total"])
    # count/hash-only mode gives the same hashes
    lean = fn(dev(mats), kmax, zero_diag=zero_diag, want_perms=False, want_residual=False, want_hashes=True)
    torch.cuda.synchronize()
    assert np.array_equal(lean["hashes"].cpu().numpy().view(np.uint64), ref["hashes"])
    assert np.array_equal(lean["counts"].cpu().numpy(), ref["counts"])


# (N <= 16, <= 32, <= 64 and > 64 take different code paths in the greedy kernel)
SHAPES = [(1, 1.0, 10), (2, 1.0, 3), (3, 0.7, 4), (5, 0.6, 2), (8, 1.0, 1000), (15, 0.9, 77), (16, 0.5, 30),
          (16, 1.0, 100000000), (17, 0.6, 50), (24, 0.4, 7), (32, 0.9, 3000), (33, 0.3, 5),
          (64, 1.0, 100000), (65, 0.4, 9), (100, 0.8, 3), (128, 0.6, 40000)]


@pytest.mark.parametrize("N,density,high", SHAPES)
@pytest.mark.parametrize("zero_diag", [False, True])
def test_greedy_random(lib, N, density, high, zero_diag):
    say("greedy random", N, density, high, zero_diag)
    mats = workloads.random_matrices(6, N, seed=900 + N, density=density, high=high)
    mats[1] = 0                                                       # an all-zero matrix in the batch
    for kmax in (3, 2 * N + 2):
        check_decomposition(lib, "greedy", mats, kmax, zero_diag)


@pytest.mark.parametrize("N,density,high", SHAPES)
@pytest.mark.parametrize("zero_diag", [False, True])
def test_bvn_random(lib, N, density, high, zero_diag):
    say("bvn random", N, density, high, zero_diag)
    nb = 6 if N <= 65 else 2
    mats = workloads.random_matrices(nb, N, seed=1900 + N, density=density, high=high)
    mats[1] = 0
    check_decomposition(lib, "bvn", mats, 5, zero_diag)
    check_decomposition(lib, "bvn", mats, oracle.bvn_bound(N) if N <= 65 else 600, zero_diag)


def test_decompose_special_cases(lib):
    say("decompose special cases")
    n = 16
    eye = np.zeros((3, n, n), dtype=np.int32)
    eye[0] = np.eye(n, dtype=np.int32)[np.random.default_rng(0).permutation(n)] * 7      # c * P
    eye[1] = 1                                                                            # all ones
    eye[2] = np.outer(np.arange(1, n + 1), np.arange(2, n + 2))                           # unique optimum
    for which in ("greedy", "bvn"):
        check_decomposition(lib, which, eye, 300, False)
        check_decomposition(lib, which, eye, 0, False)                                    # kmax = 0
    big = np.full((1, 8, 8), (1 << 28) - 1, dtype=np.int32)                               # N * max < 2^31
    check_decomposition(lib, "greedy", big, 20, False)
    check_decomposition(lib, "bvn", big, 100, False)
    with pytest.raises(lib.MoeError):
        lib.moe_decompose_greedy(torch.zeros((1, 129, 129), dtype=torch.int32, device=DEV), 4)


def test_greedy_16_bit_residual(lib):
    """How the residual is held on chip (32 bits, or 16 bits with a second launch for the matrices that do not fit)
    does not change a byte of the result."""
    say("greedy 16-bit residual")
    for N, kmax in ((5, 12), (16, 8), (64, 70), (128, 32)):
        mats = workloads.random_matrices(4, N, seed=70 + N, density=0.8, high=65536)
        mats[0, 0, 1 % N] = 65535
        mats[2, N - 1, 0] = 65536                                        # does not fit 16 bits: redone in 32
        mats[3] = mats[3] * 3                                            # most entries do not fit
        a = lib.moe_decompose_greedy(dev(mats), kmax, zero_diag=True, want_hashes=True, residual_bits=32)
        b = lib.moe_decompose_greedy(dev(mats), kmax, zero_diag=True, want_hashes=True, residual_bits=16)
        c = lib.moe_decompose_greedy(dev(mats), kmax, zero_diag=True, want_hashes=True)
        torch.cuda.synchronize()
        for key in ("perms", "durations", "counts", "residual", "hashes"):
            assert torch.equal(a[key], b[key]) and torch.equal(a[key], c[key]), (N, key)
        ref = oracle.decompose_batch("greedy", mats, kmax, zero_diag=True)
        assert np.array_equal(b["hashes"].cpu().numpy().view(np.uint64), ref["hashes"])
        assert np.array_equal(b["counts"].cpu().numpy(), ref["counts"])
    stress = workloads.stress_matrices(16, 128)
    assert stress.max() < 65536
    b = lib.moe_decompose_greedy(dev(stress), 32, zero_diag=True, want_hashes=True, residual_bits=16)
    torch.cuda.synchronize()
    ref = oracle.decompose_batch("greedy", stress, 32, zero_diag=True, nthreads=8)
    assert np.array_equal(b["hashes"].cpu().numpy().view(np.uint64), ref["hashes"])
    assert np.array_equal(b["residual"].cpu().numpy(), ref["residual"])


def test_decompose_profile_hook(lib):
    """The measurement hook records cycles, ticks and search steps per matrix and changes no result."""
    say("decompose profile hook")
    mats = workloads.random_matrices(5, 64, seed=9, density=0.8, high=5000)
    plain = lib.moe_decompose_greedy(dev(mats), 70, zero_diag=True, want_hashes=True)
    prof = torch.zeros((5, 4), dtype=torch.int64, device=DEV)
    lib.moe_decompose_profile(prof)
    try:
        timed = lib.moe_decompose_greedy(dev(mats), 70, zero_diag=True, want_hashes=True)
        torch.cuda.synchronize()
        p_greedy = prof.cpu().numpy().copy()
        lib.moe_decompose_bvn(dev(mats), 50, zero_diag=True)
        torch.cuda.synchronize()
        p_bvn = prof.cpu().numpy().copy()
    finally:
        lib.moe_decompose_profile(None)
    for key in ("perms", "durations", "counts", "residual", "hashes"):
        assert torch.equal(plain[key], timed[key]), key
    assert (p_greedy[:, 0] > 0).all() and (p_greedy[:, 1] > 0).all() and (p_greedy[:, 2] >= p_greedy[:, 3]).all() and (p_greedy[:, 3] > 0).all()
    clock_ghz = p_greedy[:, 0] / p_greedy[:, 1] * 0.1
    assert ((clock_ghz > 0.3) & (clock_ghz < 3.0)).all(), clock_ghz                 # cycles per 10 ns tick: a shader clock
    assert (p_bvn[:, 0] > 0).all() and (p_bvn[:, 2] == 0).all()
    before = prof.clone()
    lib.moe_decompose_greedy(dev(mats), 70, zero_diag=True)                       # recording is off again
    torch.cuda.synchronize()
    assert torch.equal(before, prof)


def test_mfma_probe(lib):
    """The measurement kernel runs, is timed under its name, and its accumulators hold what the loop defines: zero for
    zero operands; with varied operands every accumulator is the same product block added once per iteration, so
    twice the iterations give twice the value (up to fp32 rounding of the running sums)."""
    say("mfma probe")
    z = lib.moe_probe_mfma_bf16(0, 7, 3)
    torch.cuda.synchronize()
    assert z.shape == (3 * 256,) and bool((z == 0).all())
    lib.moe_kernel_timing_enable(True)
    a = lib.moe_probe_mfma_bf16(1, 8, 2).clone()
    b = lib.moe_probe_mfma_bf16(1, 16, 2).clone()
    torch.cuda.synchronize()
    lib.moe_kernel_timing_enable(False)
    kt = lib.moe_kernel_timing_read()
    assert kt["mfma_probe_kernel"][1] == 2 and kt["mfma_probe_kernel"][0] > 0
    assert bool(torch.isfinite(a).all()) and bool((a != 0).any())
    assert torch.allclose(b, 2 * a, rtol=1e-3, atol=1e-6)


def test_decompose_stress_matrices_128(lib):
    """The batched stress workload at its real shape (128 x 128, Zipf rows), a sample of matrices."""
    say("decompose stress 128")
    mats = workloads.stress_matrices(48, 128)
    check_decomposition(lib, "greedy", mats, 32, True)
    check_decomposition(lib, "bvn", mats[:8], 512, True)
    say("decompose stress 128: full BvN on 2 matrices")
    check_decomposition(lib, "bvn", mats[:2], oracle.bvn_bound(128), True)


def check_sinkhorn(lib, mats, kmax, zero_diag, sweeps, eps):
    """Bit-exact: both sides add in index order and divide in IEEE double precision."""
    B, N, _ = mats.shape
    out = lib.moe_decompose_sinkhorn_bvn(dev(mats), kmax, zero_diag=zero_diag, sweeps=sweeps, eps=eps)
    torch.cuda.synchronize()
    counts = out["counts"].cpu().numpy()
    perms, coef = out["perms"].cpu().numpy(), out["coeffs"].cpu().numpy()
    scaled, resid, devi = out["scaled"].cpu().numpy(), out["residual"].cpu().numpy(), out["deviation"].cpu().numpy()
    for b in range(B):
        rp, rc, rx, rr, rd = oracle.sinkhorn_bvn(mats[b], kmax=kmax, zero_diag=zero_diag, iters=sweeps, eps=eps)
        assert np.array_equal(scaled[b], rx), (N, b, np.abs(scaled[b] - rx).max())
        assert devi[b] == rd
        assert counts[b] == len(rp), (N, b, counts[b], len(rp))
        assert np.array_equal(perms[b, :len(rp)], rp), (N, b)
        assert np.array_equal(coef[b, :len(rp)], rc), (N, b)
        assert np.array_equal(resid[b], rr), (N, b)
        assert (coef[b, len(rp):] == 0).all()


@pytest.mark.parametrize("N,density,high", [(1, 1.0, 5), (2, 1.0, 3), (5, 0.7, 9), (8, 1.0, 1000), (16, 0.6, 300), (33, 0.5, 50),
                                            (64, 1.0, 5000), (65, 0.6, 20), (128, 0.7, 40000)])
@pytest.mark.parametrize("zero_diag", [False, True])
def test_sinkhorn_bvn_random(lib, N, density, high, zero_diag):
    say("sinkhorn bvn random", N, density, high, zero_diag)
    nb = 4 if N <= 65 else 2
    mats = workloads.random_matrices(nb, N, seed=2900 + N, density=density, high=high)
    mats[1] = 0
    check_sinkhorn(lib, mats, 4, zero_diag, sweeps=20, eps=1e-12)
    check_sinkhorn(lib, mats, min(N * N, 700), zero_diag, sweeps=60 if N <= 65 else 25, eps=1e-12)
    check_sinkhorn(lib, mats[:1], 10, zero_diag, sweeps=0, eps=0.5)              # no scaling at all: plain BvN steps on A


def test_sinkhorn_bvn_configs_and_errors(lib):
    say("sinkhorn bvn configs")
    for name in ("tiny", "c2", "c3"):
        cfg = workloads.CONFIGS[name]
        traffic, _ = oracle.route_histogram(workloads.config_routing(cfg), cfg.E)
        for zd in (False, True):
            check_sinkhorn(lib, traffic[None], oracle.bvn_bound(cfg.N), zd, sweeps=200, eps=1e-12)
    with pytest.raises(lib.MoeError):
        lib.moe_decompose_sinkhorn_bvn(torch.zeros((1, 4, 4), dtype=torch.int32, device=DEV), 4, sweeps=-1)
    with pytest.raises(lib.MoeError):
        lib.moe_decompose_sinkhorn_bvn(torch.zeros((1, 129, 129), dtype=torch.int32, device=DEV), 4)


# ------------------------------------------------------------------------------ slice table
@pytest.mark.parametrize("name,which", [("tiny", "greedy"), ("tiny", "bvn"), ("c2", "greedy"), ("c2", "bvn"), ("c3", "greedy")])
def test_slice_table(lib, name, which):
    say("slice table", name, which)
    cfg = workloads.CONFIGS[name]
    ids = workloads.config_routing(cfg)
    traffic, _ = oracle.route_histogram(ids, cfg.E)
    order = np.argsort(-traffic.sum(0), kind="stable")
    kmax = cfg.kmax if which == "greedy" else oracle.bvn_bound(cfg.N)
    d_ids, d_traffic = dev(ids), dev(traffic)
    fn = lib.moe_decompose_greedy if which == "greedy" else lib.moe_decompose_bvn
    sched = fn(d_traffic.unsqueeze(0), kmax, zero_diag=True)
    if which == "greedy":
        rp, rd, _ = oracle.decompose_greedy(traffic, kmax, zero_diag=True)
    else:
        rp, rd, _, _, _ = oracle.decompose_bvn(traffic, kmax, zero_diag=True)
    for r in (int(order[0]), int(order[len(order) // 2]), int(order[-1])):
        off = lib.moe_slice_table(d_ids, cfg.E, r, d_traffic, sched["perms"][0], sched["durations"][0], sched["counts"],
                                  kmax)
        torch.cuda.synchronize()
        ref, _ = oracle.slice_table(ids, cfg.E, r, traffic, rp, rd, kmax, want_rows=False)
        assert np.array_equal(off.cpu().numpy(), ref), (name, which, r)


def test_slice_table_many_windows(lib):
    """A hand-made schedule that wires one source to the receiver in thousands of matchings
    (more windows than fit in LDS) and ships one assignment at a time."""
    say("slice table many windows")
    N, E, T, topk, r = 4, 8, 6000, 1, 2
    rng = np.random.default_rng(3)
    ids = rng.integers(0, E, size=(N, T, topk)).astype(np.int32)
    traffic, _ = oracle.route_histogram(ids, E)
    kmax = 3000
    perms = np.tile(np.array([[r, 0, 1, 3]], dtype=np.uint8), (kmax, 1))      # source 0 -> r in every matching
    perms[::3] = np.array([1, r, 0, 3], dtype=np.uint8)                       # every third: source 1 -> r
    dur = rng.integers(0, 3, size=kmax).astype(np.int32)
    count = np.array([kmax - 5], dtype=np.int32)
    off = lib.moe_slice_table(dev(ids), E, r, dev(traffic), dev(perms), dev(dur), dev(count), kmax)
    torch.cuda.synchronize()
    ref, _ = oracle.slice_table(ids, E, r, traffic, perms[:kmax - 5], dur[:kmax - 5], kmax, want_rows=False)
    assert np.array_equal(off.cpu().numpy(), ref)


@pytest.mark.parametrize("name,which", [("tiny", "greedy"), ("tiny", "bvn"), ("c2", "greedy"), ("c2", "bvn"), ("c3", "greedy")])
def test_slice_table_rows(lib, name, which):
    """Row map: assignment index bit-exact with the oracle; the arrival index is the rank of that assignment among
    all assignments destined to r (sources in rank order, each in arrival order)."""
    say("slice table rows", name, which)
    cfg = workloads.CONFIGS[name]
    ids = workloads.config_routing(cfg)
    traffic, _ = oracle.route_histogram(ids, cfg.E)
    order = np.argsort(-traffic.sum(0), kind="stable")
    kmax = cfg.kmax if which == "greedy" else oracle.bvn_bound(cfg.N)
    d_ids, d_traffic = dev(ids), dev(traffic)
    if which == "greedy":
        rp, rd, _ = oracle.decompose_greedy(traffic, kmax, zero_diag=True)
    else:
        rp, rd, _, _, _ = oracle.decompose_bvn(traffic, kmax, zero_diag=True)
    pp = np.zeros((kmax, cfg.N), dtype=np.uint8)
    dd = np.zeros(kmax, dtype=np.int32)
    pp[:len(rp)], dd[:len(rd)] = rp, rd
    cnt = np.array([len(rp)], dtype=np.int32)
    for r in (int(order[0]), int(order[len(order) // 2]), int(order[-1])):
        M = int(traffic[:, r].sum())
        off, arr, asg = lib.moe_slice_table_rows(d_ids, cfg.E, r, d_traffic, dev(pp), dev(dd), dev(cnt), kmax, M)
        torch.cuda.synchronize()
        ref_off, ref_rows = oracle.slice_table(ids, cfg.E, r, traffic, rp, rd, kmax)
        assert np.array_equal(off.cpu().numpy(), ref_off), (name, which, r)
        assert np.array_equal(asg.cpu().numpy(), ref_rows), (name, which, r)
        assert np.array_equal(arr.cpu().numpy(), np.searchsorted(np.sort(ref_rows), ref_rows)), (name, which, r)
        only = lib.moe_slice_table_rows(d_ids, cfg.E, r, d_traffic, dev(pp), dev(dd), dev(cnt), kmax, M, want_assignment=False)
        torch.cuda.synchronize()
        assert only[2] is None and np.array_equal(only[1].cpu().numpy(), arr.cpu().numpy())


@pytest.mark.parametrize("T,topk", [(9001, 1), (8192, 1), (2731, 3), (5, 1), (20000, 2)])
def test_slice_table_walk_passes(lib, T, topk):
    """Assignments per source below, at and above what one pass of the walk covers, with ragged ends."""
    say("slice table walk passes T=%d topk=%d" % (T, topk))
    N, E, r = 5, 20, 3
    rng = np.random.default_rng(T + topk)
    ids = rng.integers(-2, E + 2, size=(N, T, topk)).astype(np.int32)
    traffic, _ = oracle.route_histogram(ids, E)
    kmax = 3
    rp, rd, _ = oracle.decompose_greedy(traffic, kmax, zero_diag=True)
    k = len(rd)
    perms = np.zeros((kmax, N), dtype=np.uint8); perms[:k] = rp
    dur = np.zeros(kmax, dtype=np.int32); dur[:k] = rd
    off = lib.moe_slice_table(dev(ids), E, r, dev(traffic), dev(perms), dev(dur), dev(np.array([k], dtype=np.int32)), kmax)
    torch.cuda.synchronize()
    ref, _ = oracle.slice_table(ids, E, r, traffic, rp, rd, kmax, want_rows=False)
    assert np.array_equal(off.cpu().numpy(), ref)


def test_slice_table_rows_shapes_and_errors(lib):
    say("slice table rows shapes")
    rng = np.random.default_rng(8)
    # many experts per rank (64), ids outside [0, E) are dropped, a schedule that ships in small pieces
    N, E, T, topk, r = 3, 192, 700, 3, 1
    ids = rng.integers(-5, E + 5, size=(N, T, topk)).astype(np.int32)
    traffic, _ = oracle.route_histogram(ids, E)
    kmax = 40
    perms = np.tile(np.array([[1, 2, 0]], dtype=np.uint8), (kmax, 1))          # source 0 -> r
    perms[1::2] = np.array([2, 0, 1], dtype=np.uint8)                          # every other: source 2 -> r
    dur = rng.integers(0, 30, size=kmax).astype(np.int32)
    M = int(traffic[:, r].sum())
    off, arr, asg = lib.moe_slice_table_rows(dev(ids), E, r, dev(traffic), dev(perms), dev(dur), dev(np.array([kmax - 3], dtype=np.int32)), kmax, M)
    torch.cuda.synchronize()
    ref_off, ref_rows = oracle.slice_table(ids, E, r, traffic, perms[:kmax - 3], dur[:kmax - 3], kmax)
    assert np.array_equal(off.cpu().numpy(), ref_off) and np.array_equal(asg.cpu().numpy(), ref_rows)
    assert np.array_equal(np.sort(arr.cpu().numpy()), np.arange(M))
    # too many (window, expert) counters for the row map: refused, the plain table still works
    big_k = 8192 // 64 + 1
    with pytest.raises(lib.MoeError):
        lib.moe_slice_table_rows(dev(ids), E, r, dev(traffic), dev(np.zeros((big_k, N), dtype=np.uint8)),
                                 dev(np.zeros(big_k, dtype=np.int32)), dev(np.zeros(1, dtype=np.int32)), big_k, M)


# ------------------------------------------------------------------------------ FFN
def ffn_error(y_gpu_bits, y_ref, offsets, rows=None):
    """max over (slice, expert) groups of max|y - yref| / max|yref| on the given rows."""
    y = oracle.decode_bf16(y_gpu_bits)
    if rows is None:
        rows = np.arange(int(offsets[-1]))
    grp = np.searchsorted(offsets, rows, side="right") - 1
    worst, worst_elem = 0.0, 0.0
    for g in np.unique(grp):
        sel = grp == g
        scale = np.abs(y_ref[sel]).max()
        assert scale > 0
        diff = np.abs(y[sel] - y_ref[sel])
        worst = max(worst, float(diff.max() / scale))
        # (reported beside the contract's metric: element by element, with an absolute floor of 1e-3 of the group's
        #  largest value -- a plain elementwise ratio is meaningless next to zero)
        worst_elem = max(worst_elem, float((diff / np.maximum(np.abs(y_ref[sel]), 1e-3 * scale)).max()))
    say("   (elementwise |y - ref| / max(|ref|, 1e-3 max|ref|): %.3g)" % worst_elem)
    return worst


def upload_weights(W):
    if W.dtype == "bf16":
        return dict(w_gate=dev_bf16(W.w_gate), w_up=dev_bf16(W.w_up), w_down=dev_bf16(W.w_down))
    return dict(w_gate=dev(W.w_gate), w_up=dev(W.w_up), w_down=dev(W.w_down),
                s_gate=dev(W.s_gate), s_up=dev(W.s_up), s_down=dev(W.s_down))


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("tile_rows", ["64", "128", "256"])
@pytest.mark.parametrize("E_loc,d,f,M,S", [(1, 256, 512, 700, 3), (2, 512, 384, 1500, 4), (4, 256, 128, 333, 5)])
def test_ffn_small(lib, dtype, tile_rows, E_loc, d, f, M, S):
    say("ffn small", dtype, tile_rows, E_loc, d, f, M, S)
    lib.moe_ffn_tile_override(int(tile_rows))
    try:
        W = workloads.ffn_weights(E_loc, d, f, seed=d + f, dtype=dtype)
        x = workloads.activations(M + 9, d, seed=M)                                      # 9 spare rows past the last group
        offsets = workloads.random_offsets(S * E_loc, M, seed=M + S)
        y0 = torch.full((M + 9, d), 3.0, dtype=torch.bfloat16, device=DEV)
        y = lib.moe_expert_ffn_sliced(dev_bf16(x), dev(offsets), S, E_loc, y=y0, **upload_weights(W))
        torch.cuda.synchronize()
        ref = oracle.expert_ffn_sliced(x, offsets, E_loc, W)
        yb = host_bf16_bits(y)
        check_ffn_error(ffn_error(yb[:M], ref, offsets), dtype)
        assert (oracle.decode_bf16(yb[M:]) == 3.0).all()                                  # rows past the end untouched
        # a row's result does not depend on how the rows are sliced: one slice per expert, same experts
        expert = (np.searchsorted(offsets, np.arange(M), side="right") - 1) % E_loc
        order = np.argsort(expert, kind="stable")
        off2 = np.zeros(E_loc + 1, dtype=np.int32)
        off2[1:] = np.cumsum(np.bincount(expert, minlength=E_loc))
        y2 = lib.moe_expert_ffn_sliced(dev_bf16(x[order]), dev(off2), 1, E_loc, **upload_weights(W))
        torch.cuda.synchronize()
        assert np.array_equal(host_bf16_bits(y2), yb[:M][order])
    finally:
        lib.moe_ffn_tile_override()


def test_ffn_buffers_at_addresses_with_bit_31_set(lib):
    """Output and workspace whose 64-bit addresses have bit 31 of the low word set (the kernels build buffer
    descriptors from the two halves of such addresses)."""
    say("ffn buffers above a 2 GiB boundary of the low address word")
    E_loc, d, f, M, S = 1, 256, 512, 700, 3
    W = workloads.ffn_weights(E_loc, d, f, seed=d + f)
    x = workloads.activations(M, d, seed=M)
    offsets = workloads.random_offsets(S * E_loc, M, seed=M + S)
    ws_bytes = lib.moe_ffn_workspace_bytes(M, d, f)
    y_bytes = M * d * 2
    pool = torch.empty(((1 << 32) + (64 << 20),), dtype=torch.uint8, device=DEV)
    low = pool.data_ptr() & 0xFFFFFFFF
    o = ((0x80000000 - low) % (1 << 32) + 255) // 256 * 256 + 4096
    o2 = (o + y_bytes + 255) // 256 * 256
    assert ((pool.data_ptr() + o) >> 31) & 1 and ((pool.data_ptr() + o2) >> 31) & 1 and o2 + ws_bytes <= pool.numel()
    y0 = pool[o:o + y_bytes].view(torch.bfloat16).view(M, d)
    ws = pool[o2:o2 + ws_bytes]
    for rows in ("256", "128"):
        lib.moe_ffn_tile_override(int(rows))
        try:
            y = lib.moe_expert_ffn_sliced(dev_bf16(x), dev(offsets), S, E_loc, y=y0, workspace=ws, **upload_weights(W))
            torch.cuda.synchronize()
        finally:
            lib.moe_ffn_tile_override()
        check_ffn_error(ffn_error(host_bf16_bits(y), oracle.expert_ffn_sliced(x, offsets, E_loc, W), offsets), "bf16", "rows %s" % rows)
    del pool, y0, ws, y


def test_ffn_fp8_weights_expanded_once(lib):
    """With room in the workspace and >= 2048 rows per expert the fp8 weights are expanded to bf16 before the GEMMs:
    same values, so the same result up to the order of the fp32 sums."""
    say("ffn fp8: weights expanded to bf16 once per call")
    E_loc, d, f, M, S = 2, 256, 384, 4500, 3
    W = workloads.ffn_weights(E_loc, d, f, seed=77, dtype="fp8")
    x = workloads.activations(M, d, seed=78)
    offsets = workloads.random_offsets(S * E_loc, M, seed=79)
    up = upload_weights(W)
    base = lib.moe_ffn_workspace_bytes(M, d, f)
    extra = lib.moe_ffn_expanded_weights_bytes(E_loc, d, f)
    assert extra >= 3 * E_loc * d * f * 2
    ref = oracle.expert_ffn_sliced(x, offsets, E_loc, W)
    outs = []
    for nbytes in (base, base + extra):
        ws = torch.empty((nbytes,), dtype=torch.uint8, device=DEV)
        y = lib.moe_expert_ffn_sliced(dev_bf16(x), dev(offsets), S, E_loc, workspace=ws, **up)
        torch.cuda.synchronize()
        yb = host_bf16_bits(y)
        check_ffn_error(ffn_error(yb, ref, offsets), "fp8", "workspace %d" % nbytes)
        outs.append(oracle.decode_bf16(yb))
    scale = np.abs(outs[0]).max()
    assert np.abs(outs[0] - outs[1]).max() <= 0.02 * scale


@pytest.mark.parametrize("mapped", [False, True])
def test_ffn_same_bits_every_run(lib, mapped):
    """Tiles are handed to workgroups dynamically, but the arithmetic of a tile is fixed: the output of a call
    must not change by a bit from run to run (a race inside the kernels would show here)."""
    say("ffn same bits every run", mapped)
    E_loc, d, f, S, M = 4, 1024, 768, 6, 21000
    W = workloads.ffn_weights(E_loc, d, f, seed=5, dtype="bf16")
    x = dev_bf16(workloads.activations(M, d, seed=6))
    offsets = dev(workloads.random_offsets(S * E_loc, M, seed=7))
    w = upload_weights(W)
    rng = np.random.default_rng(8)
    row_map = dev(rng.permutation(M).astype(np.int32))
    row_gate = dev(rng.random(M, dtype=np.float32))
    first = None
    for _ in range(6):
        if mapped:
            y = lib.moe_expert_ffn_sliced_mapped(x, offsets, S, E_loc, w["w_gate"], w["w_up"], w["w_down"], row_map, row_gate)
        else:
            y = lib.moe_expert_ffn_sliced(x, offsets, S, E_loc, **w)
        torch.cuda.synchronize()
        bits = y.view(torch.int16)
        if first is None:
            first = bits.clone()
        else:
            assert torch.equal(first, bits)


_MULTI = {}


def multi_tile_case(dtype):
    """36 000 rows in 6 x 4 ragged groups, d = 1536, f = 768: about 1000 tiles per phase, i.e. every workgroup runs
    several tiles and meets full blocks after full blocks, ragged ends of more and of fewer than 128 rows after either."""
    if dtype not in _MULTI:
        E_loc, d, f, S, M = 4, 1536, 768, 6, 36000
        W = workloads.ffn_weights(E_loc, d, f, seed=15, dtype=dtype)
        x = workloads.activations(M, d, seed=16)
        offsets = workloads.random_offsets(S * E_loc, M, seed=17)
        rng = np.random.default_rng(18)
        row_map = rng.permutation(M).astype(np.int32)
        gate = rng.uniform(0.05, 1.0, size=M).astype(np.float32)
        ref = oracle.expert_ffn_sliced(x, offsets, E_loc, W)
        ref_mapped, target = oracle.expert_ffn_sliced_mapped(x, offsets, E_loc, W, row_map, gate)
        _MULTI.clear()
        _MULTI[dtype] = dict(E_loc=E_loc, d=d, f=f, S=S, M=M, W=W, x=x, offsets=offsets, row_map=row_map, gate=gate, ref=ref,
                             ref_mapped=ref_mapped, target=target)
    return _MULTI[dtype]


@pytest.mark.parametrize("dtype,tile_rows,fixed", [("bf16", 0, 0), ("bf16", 0, 2), ("bf16", 256, 1), ("bf16", 128, 0), ("bf16", 64, 0),
                                                   ("fp8", 256, 0), ("fp8", 128, 0), ("fp8", 64, 0)])
def test_ffn_many_tiles_per_workgroup_all_rows(lib, dtype, tile_rows, fixed):
    """Every row against the oracle on a schedule large enough that the tile loop, the hand-over from one tile to the
    next (chained or not), ticket stealing, the counted-store wait and (both phases in one launch, the default for bf16
    weights and 256-row tiles) the wait of a phase-2 tile for its rows of h all run, for every kernel family
    (`fixed`: 0 = the call's own choice, 1 = fixed-shape kernels, 2 = adaptive-shape kernels, one launch per phase)."""
    say("ffn many tiles per workgroup", dtype, tile_rows, fixed)
    c = multi_tile_case(dtype)
    w = upload_weights(c["W"])
    sizes = np.diff(c["offsets"]) % 256
    assert ((sizes > 0) & (sizes <= 128)).any() and (sizes > 128).any() and (np.diff(c["offsets"]) >= 512).any()
    lib.moe_ffn_tile_override(tile_rows, fixed)
    try:
        x, off = dev_bf16(c["x"]), dev(c["offsets"])
        # (fp8: a workspace without room for expanded weights, so that the kernels that dequantise tile by tile run)
        ws = torch.empty((lib.moe_ffn_workspace_bytes(c["M"], c["d"], c["f"]),), dtype=torch.uint8, device=DEV)
        y = lib.moe_expert_ffn_sliced(x, off, c["S"], c["E_loc"], workspace=ws, **w)
        torch.cuda.synchronize()
        check_ffn_error(ffn_error(host_bf16_bits(y), c["ref"], c["offsets"]), dtype, "plain, all %d rows" % c["M"])
        y0 = torch.full((c["M"], c["d"]), 3.0, dtype=torch.bfloat16, device=DEV)
        ym = lib.moe_expert_ffn_sliced_mapped(x, off, c["S"], c["E_loc"], row_map=dev(c["row_map"]), row_gate=dev(c["gate"]),
                                              y=y0, workspace=ws, **w)
        torch.cuda.synchronize()
        check_ffn_error(ffn_error(host_bf16_bits(ym)[c["target"]], c["ref_mapped"], c["offsets"]), dtype, "mapped, all rows")
    finally:
        lib.moe_ffn_tile_override()


@pytest.mark.parametrize("tile_rows,fixed,panel", [(0, False, 1), (0, False, 2), (256, True, 2), (128, False, 1)])
def test_ffn_panel_walk_all_rows(lib, tile_rows, fixed, panel):
    """The tile walk in column panels (what a call chooses by itself only for experts whose weights outgrow the
    memory-side cache): 18 column units in 3 groups, walked 1 or 2 groups at a time; every row compared."""
    say("ffn panel walk", tile_rows, fixed, panel)
    E_loc, d, f, S, M = 2, 512, 2304, 3, 12000
    W = workloads.ffn_weights(E_loc, d, f, seed=25)
    x = workloads.activations(M, d, seed=26)
    offsets = workloads.random_offsets(S * E_loc, M, seed=27)
    lib.moe_ffn_tile_override(tile_rows, fixed, panel)
    try:
        y = lib.moe_expert_ffn_sliced(dev_bf16(x), dev(offsets), S, E_loc, **upload_weights(W))
        torch.cuda.synchronize()
    finally:
        lib.moe_ffn_tile_override()
    check_ffn_error(ffn_error(host_bf16_bits(y), oracle.expert_ffn_sliced(x, offsets, E_loc, W), offsets), "bf16", "all %d rows" % M)


@pytest.mark.parametrize("S,E_loc,tile_rows", [(375, 4, 0), (375, 4, 256), (1250, 4, 0), (1250, 4, 256), (5000, 1, 128)])
def test_ffn_thousands_of_groups_all_rows(lib, S, E_loc, tile_rows):
    """More (slice, expert) groups than the planning workgroup has threads (a full BvN schedule at 64 ranks has 3972
    slices): the plan is then built in several passes.  Ragged groups with empty ones; every row compared."""
    say("ffn thousands of groups", S, E_loc, tile_rows)
    d, f, M = 256, 256, 30000
    G = S * E_loc
    W = workloads.ffn_weights(E_loc, d, f, seed=G)
    x = workloads.activations(M + 3, d, seed=G + 1)
    offsets = workloads.random_offsets(G, M, seed=G + 2, empty_frac=0.3, power=12.0)     # a few groups of several tiles among crumbs
    assert (np.diff(offsets) == 0).sum() > G // 5 and (np.diff(offsets) > 256).any()
    lib.moe_ffn_tile_override(tile_rows)
    try:
        y0 = torch.full((M + 3, d), 3.0, dtype=torch.bfloat16, device=DEV)
        y = lib.moe_expert_ffn_sliced(dev_bf16(x), dev(offsets), S, E_loc, y=y0, **upload_weights(W))
        torch.cuda.synchronize()
    finally:
        lib.moe_ffn_tile_override()
    yb = host_bf16_bits(y)
    check_ffn_error(ffn_error(yb[:M], oracle.expert_ffn_sliced(x, offsets, E_loc, W), offsets), "bf16", "%d groups" % G)
    assert (oracle.decode_bf16(yb[M:]) == 3.0).all()


@pytest.mark.parametrize("tile_rows,fixed", [(0, False), (256, True), (64, False)])
def test_ffn_more_than_2_to_31_activation_elements(lib, tile_rows, fixed):
    """M * d just above 2^31 (rows are addressed with 64 bits): 8.4 M rows of 256 values in 3 x 2 groups, plain and
    through a row map; rows sampled from every group, whole tiles at the far end of the buffers included."""
    say("ffn M*d > 2^31", tile_rows, fixed)
    E_loc, d, f, S = 2, 256, 256, 3
    M = (1 << 31) // d + 4099
    assert M * d > (1 << 31)
    W = workloads.ffn_weights(E_loc, d, f, seed=41)
    w = upload_weights(W)
    offsets = workloads.random_offsets(S * E_loc, M, seed=42, empty_frac=0.0)
    x = workloads.activations_on_device(M, d, 43, DEV)
    rows = sample_rows(offsets, 300, blocks=[(M - 700, M), (offsets[3] - 300, offsets[3] + 300), (0, 256)])
    idx = torch.from_numpy(rows).to(DEV)
    g = torch.Generator(device=DEV)
    g.manual_seed(44)
    row_map = torch.randperm(M, device=DEV, generator=g).to(torch.int32)
    lib.moe_ffn_tile_override(tile_rows, fixed)
    try:
        y = lib.moe_expert_ffn_sliced(x, dev(offsets), S, E_loc, **w)
        torch.cuda.synchronize()
        ref = oracle.expert_ffn_sliced(_RowsView(host_bf16_bits(x[idx]), rows, M), offsets, E_loc, W, rows=rows)
        check_ffn_error(ffn_error(host_bf16_bits(y[idx]), ref, offsets, rows=rows), "bf16", "plain, %d sampled rows" % len(rows))
        del y
        ym = lib.moe_expert_ffn_sliced_mapped(x, dev(offsets), S, E_loc, row_map=row_map, **w)
        torch.cuda.synchronize()
        src = row_map[idx].long()                                        # arrival rows behind the sampled schedule rows
        ref = oracle.expert_ffn_sliced(_RowsView(host_bf16_bits(x[src]), rows, M), offsets, E_loc, W, rows=rows)
        check_ffn_error(ffn_error(host_bf16_bits(ym[src]), ref, offsets, rows=rows), "bf16", "mapped, %d sampled rows" % len(rows))
        del ym
    finally:
        lib.moe_ffn_tile_override()


def test_ffn_edge_cases(lib):
    say("ffn edge cases")
    E_loc, d, f = 2, 256, 128
    W = workloads.ffn_weights(E_loc, d, f, seed=1)
    up = upload_weights(W)
    x = workloads.activations(64, d, seed=2)
    # all groups empty: nothing is written
    y0 = torch.full((64, d), 5.0, dtype=torch.bfloat16, device=DEV)
    off = np.zeros(2 * E_loc + 1, dtype=np.int32)
    y = lib.moe_expert_ffn_sliced(dev_bf16(x), dev(off), 2, E_loc, y=y0, **up)
    torch.cuda.synchronize()
    assert (y.float() == 5.0).all()
    # a single row, and a group of exactly one tile plus one row
    for sizes in ([1, 0, 0, 0], [0, 0, 0, 1], [64, 0, 0, 0][::-1], [33, 31, 0, 0]):
        off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
        y = lib.moe_expert_ffn_sliced(dev_bf16(x), dev(off), 2, E_loc, **up)
        torch.cuda.synchronize()
        ref = oracle.expert_ffn_sliced(x, off, E_loc, W)
        check_ffn_error(ffn_error(host_bf16_bits(y)[:off[-1]], ref, off), "bf16", str(sizes))
    with pytest.raises(lib.MoeError):
        lib.moe_expert_ffn_sliced(dev_bf16(x[:, :128]), dev(off), 2, E_loc, w_gate=up["w_gate"][:, :, :128].contiguous(),
                                  w_up=up["w_up"][:, :, :128].contiguous(), w_down=up["w_down"][:, :128].contiguous())


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("tile_rows", ["64", "256"])
def test_ffn_mapped(lib, dtype, tile_rows):
    """Gather / scatter through a row map and the router weight in the epilogue."""
    say("ffn mapped", dtype, tile_rows)
    lib.moe_ffn_tile_override(int(tile_rows))
    try:
        E_loc, d, f, M, S = 2, 512, 384, 1500, 4
        rng = np.random.default_rng(77)
        W = workloads.ffn_weights(E_loc, d, f, seed=5, dtype=dtype)
        x = workloads.activations(M, d, seed=6)                                          # arrival order
        offsets = workloads.random_offsets(S * E_loc, M - 40, seed=7)                    # 40 arrival rows are never scheduled
        used = int(offsets[-1])
        row_map = rng.permutation(M)[:used].astype(np.int32)
        gate = rng.uniform(0.05, 1.0, size=used).astype(np.float32)
        y0 = torch.full((M, d), 3.0, dtype=torch.bfloat16, device=DEV)
        y = lib.moe_expert_ffn_sliced_mapped(dev_bf16(x), dev(offsets), S, E_loc, row_map=dev(row_map), row_gate=dev(gate),
                                             y=y0, **upload_weights(W))
        torch.cuda.synchronize()
        ref, target = oracle.expert_ffn_sliced_mapped(x, offsets, E_loc, W, row_map, gate)
        yb = host_bf16_bits(y)
        check_ffn_error(ffn_error(yb[target], ref, offsets), dtype)
        untouched = np.setdiff1d(np.arange(M), target)
        assert (oracle.decode_bf16(yb[untouched]) == 3.0).all()
        # identity map and unit gate: the very bytes of the plain call
        ident = np.arange(used, dtype=np.int32)
        ya = lib.moe_expert_ffn_sliced_mapped(dev_bf16(x), dev(offsets), S, E_loc, row_map=dev(ident),
                                              row_gate=dev(np.ones(used, dtype=np.float32)), **upload_weights(W))
        yp = lib.moe_expert_ffn_sliced(dev_bf16(x), dev(offsets), S, E_loc, **upload_weights(W))
        torch.cuda.synchronize()
        assert np.array_equal(host_bf16_bits(ya)[:used], host_bf16_bits(yp)[:used])
        # gathering through the map equals running the plain call on rows gathered beforehand
        yg = lib.moe_expert_ffn_sliced(dev_bf16(np.ascontiguousarray(x[row_map])), dev(offsets), S, E_loc, **upload_weights(W))
        ym = lib.moe_expert_ffn_sliced_mapped(dev_bf16(x), dev(offsets), S, E_loc, row_map=dev(row_map), **upload_weights(W))
        torch.cuda.synchronize()
        assert np.array_equal(host_bf16_bits(ym)[row_map], host_bf16_bits(yg)[:used])
    finally:
        lib.moe_ffn_tile_override()


# ------------------------------------------------------------------------------ FFN backward
def check_backward(lib, E_loc, d, f, M, S, seed, what, spare=0, empty_frac=0.15):
    W = workloads.ffn_weights(E_loc, d, f, seed=seed)
    x = workloads.activations(M + spare, d, seed=seed + 1)
    dy = workloads.activations(M + spare, d, seed=seed + 2)
    offsets = workloads.random_offsets(S * E_loc, M, seed=seed + 3, empty_frac=empty_frac)
    w = upload_weights(W)
    out = lib.moe_expert_ffn_backward_sliced(dev_bf16(x), dev_bf16(dy), dev(offsets), S, E_loc, w["w_gate"], w["w_up"], w["w_down"])
    torch.cuda.synchronize()
    dx, dWg, dWu, dWd = oracle.expert_ffn_backward_sliced(x, dy, offsets, E_loc, W)
    if M > 0:
        check_ffn_error(ffn_error(host_bf16_bits(out["dx"])[:M], dx, offsets), "bf16", what + " dx")
    for name, ref in (("dw_gate", dWg), ("dw_up", dWu), ("dw_down", dWd)):
        got = oracle.decode_bf16(host_bf16_bits(out[name]))
        for e in range(E_loc):
            scale = np.abs(ref[e]).max()
            if scale == 0:
                assert not got[e].any(), (name, e)
                continue
            check_ffn_error(float(np.abs(got[e] - ref[e]).max() / scale), "bf16", "%s %s[%d]" % (what, name, e))
    return out


@pytest.mark.parametrize("E_loc,d,f,M,S", [(1, 256, 256, 300, 1), (2, 256, 384, 1500, 3), (4, 512, 640, 5000, 4), (3, 256, 1408, 900, 2)])
def test_ffn_backward_small(lib, E_loc, d, f, M, S):
    """dx for every row and the three weight gradients of every expert against the float64 chain rule."""
    say("ffn backward small", E_loc, d, f, M, S)
    check_backward(lib, E_loc, d, f, M, S, seed=d + f + M, what="small", spare=5)


def test_ffn_backward_edge_cases(lib):
    say("ffn backward edge cases")
    # an expert without rows (zero weight gradients), a single row, no rows at all
    E_loc, d, f = 3, 256, 256
    W = workloads.ffn_weights(E_loc, d, f, seed=3)
    w = upload_weights(W)
    x = workloads.activations(40, d, seed=4)
    dy = workloads.activations(40, d, seed=5)
    for sizes in ([40, 0, 0], [0, 1, 0], [0, 0, 0], [13, 0, 27]):
        off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
        out = lib.moe_expert_ffn_backward_sliced(dev_bf16(x), dev_bf16(dy), dev(off), 1, E_loc, w["w_gate"], w["w_up"], w["w_down"])
        torch.cuda.synchronize()
        dx, dWg, dWu, dWd = oracle.expert_ffn_backward_sliced(x, dy, off, E_loc, W)
        n = int(off[-1])
        if n:
            check_ffn_error(ffn_error(host_bf16_bits(out["dx"])[:n], dx, off), "bf16", str(sizes))
        for name, ref in (("dw_gate", dWg), ("dw_up", dWu), ("dw_down", dWd)):
            got = oracle.decode_bf16(host_bf16_bits(out[name]))
            for e in range(E_loc):
                if sizes[e] == 0:
                    assert not got[e].any(), (sizes, name, e)
                else:
                    assert np.abs(got[e] - ref[e]).max() <= FFN_GUARD["bf16"] * np.abs(ref[e]).max(), (sizes, name, e)
    with pytest.raises(lib.MoeError):                                    # f below the smallest supported width
        lib.moe_expert_ffn_backward_sliced(dev_bf16(x), dev_bf16(dy), dev(off), 1, E_loc, w["w_gate"][:, :128].contiguous(),
                                           w["w_up"][:, :128].contiguous(), w["w_down"][:, :, :128].contiguous())


def test_ffn_backward_many_tiles(lib):
    """A schedule on which every workgroup runs several tiles in each of the six matrix launches."""
    say("ffn backward many tiles")
    check_backward(lib, 4, 1536, 768, 36000, 6, seed=61, what="36000 rows")


def test_whole_path_backward_c2(lib):
    """c2's hottest receiving rank: the schedule from the GPU path, then the backward pass of its FFN; every row of dx and
    all twelve weight gradients against the oracle."""
    say("whole path backward c2")
    cfg = workloads.CONFIGS["c2"]
    ids = workloads.config_routing(cfg)
    d_ids = dev(ids)
    traffic, _ = lib.moe_route_histogram(d_ids, cfg.E)
    r = int(traffic.sum(0).argmax().item())
    sched = lib.moe_decompose_greedy(traffic.unsqueeze(0), cfg.kmax, zero_diag=True)
    offsets = lib.moe_slice_table(d_ids, cfg.E, r, traffic, sched["perms"][0], sched["durations"][0], sched["counts"], cfg.kmax)
    torch.cuda.synchronize()
    off = offsets.cpu().numpy()
    M = int(off[-1])
    W, Wd = config_weights(cfg)
    x = workloads.activations(M, cfg.d, seed=cfg.seed + 3)
    dy = workloads.activations(M, cfg.d, seed=cfg.seed + 4)
    out = lib.moe_expert_ffn_backward_sliced(dev_bf16(x), dev_bf16(dy), offsets, cfg.kmax + 2, cfg.E_loc, Wd["w_gate"], Wd["w_up"], Wd["w_down"])
    torch.cuda.synchronize()
    dx, dWg, dWu, dWd = oracle.expert_ffn_backward_sliced(x, dy, off, cfg.E_loc, W)
    check_ffn_error(ffn_error(host_bf16_bits(out["dx"]), dx, off), "bf16", "dx, all %d rows" % M)
    for name, ref in (("dw_gate", dWg), ("dw_up", dWu), ("dw_down", dWd)):
        got = oracle.decode_bf16(host_bf16_bits(out[name]))
        for e in range(cfg.E_loc):
            check_ffn_error(float(np.abs(got[e] - ref[e]).max() / np.abs(ref[e]).max()), "bf16", "%s[%d]" % (name, e))
    _WEIGHTS.clear()


# ------------------------------------------------------------------------------ combine
def combine_tolerance(y_bits, row_of, gate, ref):
    """fp32 accumulation of topk terms (2^-24 of the terms' magnitudes each) and one rounding to bf16 (2^-9 of the
    result): |out - ref| <= 2^-8 |ref| + 2^-20 sum_j |gate * y| elementwise, with room to spare."""
    y = np.abs(oracle.decode_bf16(y_bits))
    live = (row_of >= 0) & (row_of < y.shape[0])
    g = np.ones(row_of.shape, dtype=np.float64) if gate is None else np.abs(gate.astype(np.float64))
    mag = (y[np.clip(row_of, 0, y.shape[0] - 1)] * (g * live)[:, :, None]).sum(axis=1)
    return 2.0 ** -8 * np.abs(ref) + 2.0 ** -20 * mag + 1e-30


@pytest.mark.parametrize("T,topk,d,R", [(1, 1, 8, 1), (37, 2, 256, 80), (50, 3, 2056, 160), (19, 8, 4096, 200), (300, 4, 7168, 1200),
                                       (11, 6, 512, 70), (5, 5, 16, 40)])
@pytest.mark.parametrize("gated", [True, False])
def test_combine_topk_sum(lib, T, topk, d, R, gated):
    say("combine", T, topk, d, R, gated)
    rng = np.random.default_rng(T * 31 + topk)
    y = workloads.activations(R, d, seed=T + d)
    row_of = rng.integers(0, R, size=(T, topk)).astype(np.int32)
    if T > 4:
        row_of[1, 0] = -1                                              # a dropped assignment
        row_of[2, :] = -1                                              # a token that lost every expert
        row_of[3, topk - 1] = R + 5                                    # past the end: ignored as well
    gate = rng.uniform(0.0, 1.0, size=(T, topk)).astype(np.float32) if gated else None
    out0 = torch.full((T, d), 3.0, dtype=torch.bfloat16, device=DEV)
    out = lib.moe_combine_topk_sum(dev_bf16(y), dev(row_of), dev(gate) if gated else None, out=out0)
    torch.cuda.synchronize()
    ref = oracle.combine_topk_sum(y, row_of, gate)
    got = oracle.decode_bf16(host_bf16_bits(out))
    assert (np.abs(got - ref) <= combine_tolerance(y, row_of, gate, ref)).all(), np.abs(got - ref).max()
    if T > 4:
        assert not got[2].any()


def test_moe_layer_dispatch_compute_combine(lib):
    """One whole layer on one GPU (every expert local): tokens -> one row per (token, expert) assignment -> slice table
    with row map -> FFN with fused gather, scatter and router weight -> weighted top-k sum per token; against
    sum_j gate[t][j] * FFN_{e(t,j)}(x_t) evaluated by the oracle."""
    say("moe layer: dispatch -> compute -> combine")
    T, E, topk, d, f = 3000, 4, 2, 512, 384
    ids = workloads.route_topk(1, T, E, topk, 1.0, seed=77)
    rng = np.random.default_rng(78)
    gate = rng.uniform(0.1, 1.0, size=(T, topk)).astype(np.float32)
    W = workloads.ffn_weights(E, d, f, seed=79)
    x_tok = workloads.activations(T, d, seed=80)
    x_arr = np.repeat(x_tok, topk, axis=0)                               # arrival order: (token, slot)
    d_ids = dev(ids)
    traffic, _ = lib.moe_route_histogram(d_ids, E)
    kmax = 2
    sched = lib.moe_decompose_greedy(traffic.unsqueeze(0), kmax, zero_diag=True)
    M = T * topk
    offsets, arr, asg = lib.moe_slice_table_rows(d_ids, E, 0, traffic, sched["perms"][0], sched["durations"][0], sched["counts"], kmax, M)
    torch.cuda.synchronize()
    assert int(offsets[-1].item()) == M and torch.equal(arr, asg)        # one source: arrival index = assignment index
    row_gate = dev(gate.reshape(-1))[arr.long()].contiguous()            # router weight of the assignment behind each schedule row
    y_arr = lib.moe_expert_ffn_sliced_mapped(dev_bf16(x_arr), offsets, kmax + 2, E, row_map=arr, row_gate=row_gate, **upload_weights(W))
    row_of = np.arange(M, dtype=np.int32).reshape(T, topk)
    out = lib.moe_combine_topk_sum(y_arr, dev(row_of))
    torch.cuda.synchronize()
    # oracle: every assignment through its expert, then the weighted sum
    off_e = np.zeros(E + 1, dtype=np.int32)
    flat = ids.reshape(-1)
    order = np.argsort(flat, kind="stable")
    off_e[1:] = np.cumsum(np.bincount(flat, minlength=E))
    y_sorted = oracle.expert_ffn_sliced(x_arr[order], off_e, E, W)
    y_asg = np.empty_like(y_sorted)
    y_asg[order] = y_sorted
    ref = (y_asg.reshape(T, topk, d) * gate.astype(np.float64)[:, :, None]).sum(axis=1)
    got = oracle.decode_bf16(host_bf16_bits(out))
    err = float(np.abs(got - ref).max() / np.abs(ref).max())
    check_ffn_error(err, "bf16", "layer output, %d tokens" % T)


def sample_rows(off, per_group, seed=1, blocks=()):
    """Every non-empty group contributes its first and last rows plus a random sample; `blocks` adds every row of the
    given (first row, end row) stretches."""
    rng = np.random.default_rng(seed)
    off = np.asarray(off, dtype=np.int64)
    rows = []
    for g in range(len(off) - 1):
        lo, hi = off[g], off[g + 1]
        if hi > lo:
            rows += [lo, hi - 1] + list(rng.integers(lo, hi, size=min(per_group, hi - lo)))
    for lo, hi in blocks:
        rows += list(range(int(lo), int(hi)))
    return np.unique(np.array(rows, dtype=np.int64))


def whole_tiles(off, want, tile=256):
    """Row stretches covering whole 256-row tiles: the first tile of every large group, a tile from the middle of the
    largest group, and the ragged last tiles of the groups -- `want` stretches in all (fewer if the schedule is small)."""
    off = np.asarray(off, dtype=np.int64)
    size = np.diff(off)
    firsts = [(off[g], min(off[g] + tile, off[g + 1])) for g in np.argsort(-size, kind="stable") if size[g] >= tile]
    tails = [(off[g] + (size[g] - 1) // tile * tile, off[g + 1]) for g in np.argsort(-size, kind="stable") if size[g] > tile and size[g] % tile]
    g = int(np.argmax(size))
    mid = [(off[g] + size[g] // tile // 2 * tile, min(off[g] + (size[g] // tile // 2 + 1) * tile, off[g + 1]))] if size[g] >= 3 * tile else []
    out, k = [], 0
    while len(out) < want and (k < len(firsts) or k < len(tails) or k < len(mid)):
        for lst in (firsts, tails, mid):
            if k < len(lst) and len(out) < want:
                out.append(lst[k])
        k += 1
    return out


def test_whole_path_with_row_map_c2(lib):
    """c2 at full size: rows arrive source by source; slice table -> row map -> FFN with fused gather / scatter.
    Every row is compared."""
    say("whole path with row map, c2")
    cfg = workloads.CONFIGS["c2"]
    ids = workloads.config_routing(cfg)
    d_ids = dev(ids)
    traffic, _ = lib.moe_route_histogram(d_ids, cfg.E)
    r = int(traffic.sum(0).argmax().item())
    sched = lib.moe_decompose_greedy(traffic.unsqueeze(0), cfg.kmax, zero_diag=True)
    M = int(traffic[:, r].sum().item())
    offsets, arr, asg = lib.moe_slice_table_rows(d_ids, cfg.E, r, traffic, sched["perms"][0], sched["durations"][0],
                                                 sched["counts"], cfg.kmax, M)
    W = workloads.ffn_weights(cfg.E_loc, cfg.d, cfg.f, seed=cfg.seed, dtype=cfg.weight_dtype)
    x = workloads.activations(M, cfg.d, seed=cfg.seed + 1)                                # arrival order
    gate = np.random.default_rng(5).uniform(0.05, 1.0, size=M).astype(np.float32)
    y = lib.moe_expert_ffn_sliced_mapped(dev_bf16(x), offsets, cfg.kmax + 2, cfg.E_loc, row_map=arr, row_gate=dev(gate),
                                         **upload_weights(W))
    torch.cuda.synchronize()
    th = traffic.cpu().numpy()
    rp, rd, _ = oracle.decompose_greedy(th, cfg.kmax, zero_diag=True)
    ref_off, ref_rows = oracle.slice_table(ids, cfg.E, r, th, rp, rd, cfg.kmax)
    assert np.array_equal(offsets.cpu().numpy(), ref_off) and np.array_equal(asg.cpu().numpy(), ref_rows)
    row_map = np.searchsorted(np.sort(ref_rows), ref_rows)
    ref, target = oracle.expert_ffn_sliced_mapped(x, ref_off, cfg.E_loc, W, row_map, gate)
    assert np.array_equal(np.sort(target), np.arange(M))
    check_ffn_error(ffn_error(host_bf16_bits(y)[target], ref, ref_off), "bf16", "all %d rows" % M)


# ------------------------------------------------------------------------------ whole path, full-size configs
_WEIGHTS = {}


def config_weights(cfg):
    """(host weights, uploaded weights) of a named config, drawn once per test session (the fp8 set takes half a minute)."""
    if cfg.name not in _WEIGHTS:
        W = workloads.ffn_weights(cfg.E_loc, cfg.d, cfg.f, seed=cfg.seed, dtype=cfg.weight_dtype)
        _WEIGHTS.clear()                                              # one set at a time on the device
        _WEIGHTS[cfg.name] = (W, upload_weights(W))
    return _WEIGHTS[cfg.name]


def test_whole_path_under_graph_capture(lib):
    """The library allocates nothing, copies nothing and clears nothing with runtime calls, so histogram -> greedy ->
    slice table (on the built-in work area) -> FFN can be recorded into a HIP graph once, with the row capacity as M
    (rows past offsets[last] are left alone), and replayed on new routings and activations.  Every replay is compared
    bit for bit with the same calls made eagerly on the same inputs (eager work and synchronisation between replays)."""
    say("whole path under graph capture")
    cfg = workloads.CONFIGS["tiny"]
    N, E, kmax, r = cfg.N, cfg.E, cfg.kmax, 3
    cap = N * cfg.T * cfg.topk                                         # no routing sends more rows than this to one rank
    W, Wd = config_weights(cfg)
    ids_s = torch.zeros((N, cfg.T, cfg.topk), dtype=torch.int32, device=DEV)
    x_s = torch.zeros((cap, cfg.d), dtype=torch.bfloat16, device=DEV)
    y_s = torch.zeros((cap, cfg.d), dtype=torch.bfloat16, device=DEV)
    traffic = torch.zeros((N, N), dtype=torch.int32, device=DEV)
    counts_e = torch.zeros((N, E), dtype=torch.int32, device=DEV)
    sched = dict(perms=torch.zeros((1, kmax, N), dtype=torch.uint8, device=DEV), durations=torch.zeros((1, kmax), dtype=torch.int32, device=DEV),
                 counts=torch.zeros((1,), dtype=torch.int32, device=DEV), residual=torch.zeros((1, N, N), dtype=torch.int32, device=DEV), hashes=None)
    offsets = torch.zeros(((kmax + 2) * cfg.E_loc + 1,), dtype=torch.int32, device=DEV)
    ws = torch.empty((lib.moe_ffn_workspace_bytes(cap, cfg.d, cfg.f),), dtype=torch.uint8, device=DEV)

    def path():
        lib.moe_route_histogram(ids_s, E, traffic=traffic, expert_counts=counts_e)
        lib.moe_decompose_greedy(traffic.view(1, N, N), kmax, zero_diag=True, out=sched)
        lib.moe_slice_table_static(ids_s, E, r, traffic, sched["perms"][0], sched["durations"][0], sched["counts"], kmax, offsets)
        lib.moe_expert_ffn_sliced(x_s, offsets, kmax + 2, cfg.E_loc, y=y_s, workspace=ws, **Wd)

    def load_inputs(seed):
        rng = np.random.default_rng(seed)
        ids_s.copy_(torch.from_numpy(rng.integers(0, E, size=(N, cfg.T, cfg.topk), dtype=np.int32)))
        x_s.copy_(workloads.activations_on_device(cap, cfg.d, 100 + seed, DEV))

    def clear():
        for t in (traffic, sched["perms"], sched["durations"], sched["counts"], sched["residual"], offsets):
            t.zero_()
        y_s.fill_(0.5)

    outputs = lambda: [t.clone() for t in (traffic, sched["perms"], sched["durations"], sched["counts"], sched["residual"], offsets, y_s)]
    load_inputs(0)
    path()                                                             # warm-up outside the capture (per-device kernel attributes)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        path()
    for seed in (1, 2, 3):
        load_inputs(seed)
        clear()
        path()
        torch.cuda.synchronize()
        eager = outputs()
        clear()                                                         # (entries past counts / offsets[last] are left alone by the calls)
        graph.replay()
        torch.cuda.synchronize()
        for name, a, b in zip(("traffic", "perms", "durations", "counts", "residual", "offsets", "y"), eager, outputs()):
            assert torch.equal(a, b), (seed, name)
        M = int(offsets[-1].item())
        assert 0 < M < cap and bool((y_s[M:] == 0.5).all())                 # rows past the schedule are untouched
    # one replay against the oracle as well (the eager path is what the other tests compare with it)
    off = offsets.cpu().numpy().astype(np.int64)
    rows = np.arange(int(off[-1]), dtype=np.int64)
    ref = oracle.expert_ffn_sliced(host_bf16_bits(x_s[: int(off[-1])]), off, cfg.E_loc, W, rows=rows)
    check_ffn_error(ffn_error(host_bf16_bits(y_s[: int(off[-1])]), ref, off, rows=rows), cfg.weight_dtype, "graph replay")


def run_path(lib, cfg, r, which="greedy", x_seed=0, x_on_device=False):
    """histogram -> decomposition -> slice table -> FFN on the GPU; returns everything on the host (x and y stay on
    the device when x_on_device: the checker reads back the rows it compares)."""
    ids = workloads.config_routing(cfg)
    d_ids = dev(ids)
    traffic, _ = lib.moe_route_histogram(d_ids, cfg.E)
    kmax = cfg.kmax if which == "greedy" else oracle.bvn_bound(cfg.N)
    fn = lib.moe_decompose_greedy if which == "greedy" else lib.moe_decompose_bvn
    sched = fn(traffic.unsqueeze(0), kmax, zero_diag=True)
    offsets = lib.moe_slice_table(d_ids, cfg.E, r, traffic, sched["perms"][0], sched["durations"][0], sched["counts"], kmax)
    torch.cuda.synchronize()
    M = int(offsets[-1].item())
    W, Wd = config_weights(cfg)
    if x_on_device:
        x = workloads.activations_on_device(M, cfg.d, cfg.seed + x_seed, DEV)
        xd = x
    else:
        x = workloads.activations(M, cfg.d, seed=cfg.seed + x_seed)
        xd = dev_bf16(x)
    say("   rows", M, "FFN call")
    y = lib.moe_expert_ffn_sliced(xd, offsets, kmax + 2, cfg.E_loc, **Wd)
    torch.cuda.synchronize()
    return dict(ids=ids, traffic=traffic.cpu().numpy(), sched={k: (v.cpu().numpy() if v is not None else None) for k, v in sched.items()},
                offsets=offsets.cpu().numpy(), M=M, W=W, x=x, y=y if x_on_device else host_bf16_bits(y), kmax=kmax)


def check_path(cfg, r, res, which, per_group=None, tiles=0):
    """Integer stages bit-exact; FFN on every row (per_group None) or on a sample: per_group random rows of every group,
    its first and last row, and every row of `tiles` whole 256-row tiles."""
    traffic, _ = oracle.route_histogram(res["ids"], cfg.E)
    assert np.array_equal(res["traffic"], traffic)
    kmax = res["kmax"]
    if which == "greedy":
        rp, rd, rr = oracle.decompose_greedy(traffic, kmax, zero_diag=True)
    else:
        rp, rd, rr, _, _ = oracle.decompose_bvn(traffic, kmax, zero_diag=True)
    c = int(res["sched"]["counts"][0])
    assert c == len(rd)
    assert np.array_equal(res["sched"]["perms"][0, :c], rp) and np.array_equal(res["sched"]["durations"][0, :c], rd)
    assert np.array_equal(res["sched"]["residual"][0], rr)
    ref_off, _ = oracle.slice_table(res["ids"], cfg.E, r, traffic, rp, rd, kmax, want_rows=False)
    assert np.array_equal(res["offsets"], ref_off)
    assert res["M"] == traffic[:, r].sum()
    off = res["offsets"].astype(np.int64)
    if per_group is None:
        rows = np.arange(res["M"], dtype=np.int64)
    else:
        rows = sample_rows(off, per_group, blocks=whole_tiles(off, tiles))
    if torch.is_tensor(res["x"]):                                     # x, y on the device: fetch the compared rows only
        idx = torch.from_numpy(rows).to(DEV)
        x_rows, y_rows = host_bf16_bits(res["x"][idx]), host_bf16_bits(res["y"][idx])
        ref = oracle.expert_ffn_sliced(_RowsView(x_rows, rows, res["M"]), off, cfg.E_loc, res["W"], rows=rows)
    else:
        y_rows = res["y"][rows]
        ref = oracle.expert_ffn_sliced(res["x"], off, cfg.E_loc, res["W"], rows=rows)
    check_ffn_error(ffn_error(y_rows, ref, off, rows=rows), cfg.weight_dtype, "%d of %d rows" % (len(rows), res["M"]))


class _RowsView:
    """Stands in for x[M][d] when only some rows are on the host: indexing with a subset of `rows` returns them."""
    def __init__(self, data, rows, M):
        self.data, self.rows, self.shape = data, rows, (M, data.shape[1])

    def __getitem__(self, idx):
        pos = np.searchsorted(self.rows, idx)
        assert np.array_equal(self.rows[pos], idx)
        return self.data[pos]


@pytest.mark.parametrize("name,which", [("tiny", "greedy"), ("tiny", "bvn"), ("c2", "greedy"), ("c2", "bvn")])
def test_whole_path_full_size(lib, name, which):
    """Hottest receiving rank (the rank the bench runs), every row compared."""
    cfg = workloads.CONFIGS[name]
    say("whole path", name, which)
    ids = workloads.config_routing(cfg)
    traffic, _ = oracle.route_histogram(ids, cfg.E)
    r = int(np.argmax(traffic.sum(0)))
    res = run_path(lib, cfg, r, which)
    check_path(cfg, r, res, which)


def test_whole_path_c3_hottest_rank(lib):
    """The 14336-wide expert on its hottest receiving rank (72 408 rows, the bench workload): at least 256 rows of every
    group and every row of 10 whole tiles."""
    cfg = workloads.CONFIGS["c3"]
    say("whole path c3, hottest rank")
    ids = workloads.config_routing(cfg)
    traffic, _ = oracle.route_histogram(ids, cfg.E)
    r = int(np.argmax(traffic.sum(0)))
    res = run_path(lib, cfg, r, "greedy")
    assert res["M"] == traffic[:, r].sum() and res["M"] > 70000
    check_path(cfg, r, res, "greedy", per_group=256, tiles=10)


@pytest.mark.parametrize("rank", ["median", "hottest"])
def test_whole_path_c4_fp8(lib, rank):
    """64 ranks, 256 experts, top-8, heavy skew, fp8 block-scaled weights.  The hottest receiving rank gets 529 867 rows
    (7.6 GB of activations: M * d > 2^31, drawn on the device); rows of every (slice, expert) group are compared."""
    cfg = workloads.CONFIGS["c4"]
    say("whole path c4 fp8,", rank, "rank")
    ids = workloads.config_routing(cfg)
    traffic, _ = oracle.route_histogram(ids, cfg.E)
    order = np.argsort(-traffic.sum(0), kind="stable")
    r = int(order[0]) if rank == "hottest" else int(order[len(order) // 2])
    res = run_path(lib, cfg, r, "greedy", x_on_device=(rank == "hottest"))
    if rank == "hottest":
        assert res["M"] * cfg.d > (1 << 31)
        check_path(cfg, r, res, "greedy", per_group=40, tiles=4)
    else:
        check_path(cfg, r, res, "greedy", per_group=16, tiles=2)
    _WEIGHTS.clear()


def test_decompose_stress_batch_hashes(lib):
    """A larger slice of the batched stress workload in count/hash-only mode: every schedule hash equals the
    oracle's, and the full batch size runs with sane counts."""
    say("decompose stress batch hashes")
    mats = workloads.stress_matrices(1024, 128)
    # (a batch this large takes the 16-bit residual by itself; two matrices get entries that do not fit and are redone)
    mats[5, 3, 77] = 70000
    mats[700] = mats[700] * 2
    assert mats[700].max() >= 65536
    out = lib.moe_decompose_greedy(dev(mats), 32, zero_diag=True, want_perms=False, want_residual=False, want_hashes=True)
    torch.cuda.synchronize()
    ref = oracle.decompose_batch("greedy", mats, 32, zero_diag=True, nthreads=16, want_perms=False, want_residual=False)
    assert np.array_equal(out["counts"].cpu().numpy(), ref["counts"])
    assert np.array_equal(out["hashes"].cpu().numpy().view(np.uint64), ref["hashes"])
    assert np.array_equal(out["durations"].cpu().numpy(), ref["durations"])
    big = torch.from_numpy(np.tile(mats, (8, 1, 1))).to(DEV)                 # 8192 matrices, the stress batch size
    out8 = lib.moe_decompose_greedy(big, 32, zero_diag=True, want_perms=False, want_residual=False, want_hashes=True)
    torch.cuda.synchronize()
    assert np.array_equal(out8["hashes"].cpu().numpy().view(np.uint64), np.tile(ref["hashes"], 8))

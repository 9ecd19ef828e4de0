#!/usr/bin/env python3
"""Benchmark of the MoE circuit-schedule hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic routing:
    routing histogram -> greedy max-weight decomposition (cap kmax)      [main stream]
                      -> Birkhoff-von Neumann baseline decomposition     [second stream, joined at step end]
                      -> slice table of the receiving rank -> sliced expert SwiGLU FFN
All inputs (router ids, weights, grouped activations) are resident in HBM before the timed
region.  Prints ONE JSON line.  `value` = algorithmic FFN flops of the step / whole step time.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2", choices=["tiny", "c2", "c3"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 256 MiB device-to-device copy (reference reading for HBM byte counters)")
    ap.add_argument("--summarize-counters", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"),
                    help="no GPU work: turn the counter_collection.csv files of the two rocprofv3 --pmc runs (FETCH_SIZE, "
                         "WRITE_SIZE; both with --calibration-copy) into profiles/ffn_<workload>_hbm_traffic.{md,json}")
    return ap.parse_args()


def code_digest(path):
    """SHA-256 of a source file without its // comments and blank space: a stored counter figure stays valid across
    edits that cannot change the kernel."""
    import hashlib, re
    lines = []
    for line in open(path, encoding="utf-8"):
        line = re.sub(r"//.*$", "", line).strip()
        if line:
            lines.append(re.sub(r"\s+", " ", line))
    return hashlib.sha256("\n".join(lines).encode()).hexdigest()


def summarize_counters(workload, fetch_csv, write_csv):
    """FETCH_SIZE / WRITE_SIZE (KiB per dispatch) of the two FFN kernels, scaled by what the same counter reads for the
    256 MiB calibration copy; stored with the SHA-256 of the kernel source it was measured on."""
    import collections
    import csv
    import hashlib

    def averages(path):
        acc = collections.defaultdict(list)
        for row in csv.DictReader(open(path)):
            k = row["Kernel_Name"]
            key = ("ffn_gemm1_kernel" if "ffn_adaptive_kernel<1>" in k or "ffn_gemm_kernel<1," in k else
                   "ffn_gemm2_kernel" if "ffn_adaptive_kernel<2>" in k or "ffn_gemm_kernel<2," in k else
                   "copy" if "copyBuffer" in k else None)
            if key:
                acc[key].append(float(row["Counter_Value"]))
        return {k: (max(v) if k == "copy" else sum(v) / len(v)) for k, v in acc.items()}     # the copy: its largest dispatch

    f, w = averages(fetch_csv), averages(write_csv)
    cal_f, cal_w = 262144.0 / f["copy"], 262144.0 / w["copy"]
    detail = {}
    for k in ("ffn_gemm1_kernel", "ffn_gemm2_kernel"):
        rb, wb = f[k] * cal_f * 1024, w[k] * cal_w * 1024
        detail[k] = {"read_bytes": rb, "write_bytes": wb, "total_bytes": rb + wb}
    rel = "paper_2605_26845_amd/csrc/ffn.hip"
    sha = code_digest(os.path.join(ROOT, rel))
    base = os.path.join(ROOT, "profiles", "ffn_%s_hbm_traffic" % workload)
    json.dump({"kernel": "ffn_gemm1_kernel", "workload": workload, "source_sha256": {rel: sha},
               "traffic_bytes_per_launch": detail["ffn_gemm1_kernel"]["total_bytes"], "detail": detail,
               "see": "profiles/ffn_%s_hbm_traffic.md" % workload}, open(base + ".json", "w"), indent=1)
    lines = ["# HBM-side byte counters (rocprofv3 --pmc), bench.py workload %s, the two FFN kernels (gemm1 = phase 1: gate/up + SwiGLU)" % workload,
             "", "Commands (run from the repository root with TMPDIR=/tmp on the MI355X box, one counter per run; then the summary, no GPU needed):", ""]
    rel_csv = [os.path.relpath(os.path.abspath(c), ROOT) for c in (fetch_csv, write_csv)]      # as given on the command line
    for c, path in zip(("FETCH_SIZE", "WRITE_SIZE"), rel_csv):
        lines.append("    rocprofv3 --pmc %s --output-format csv -d %s -o p -- python3 bench.py --workload %s --steps 10 "
                     "--warmup 2 --no-extras --no-cpu-baseline --calibration-copy" % (c, os.path.dirname(path), workload))
    lines += ["    python3 bench.py --workload %s --summarize-counters %s %s" % (workload, rel_csv[0], rel_csv[1]), "",
              "Calibration: the plain device-to-device copy of 256 MiB (`--calibration-copy`, the largest __amd_rocclr_copyBuffer dispatch) reads",
              "FETCH_SIZE = %.1f and WRITE_SIZE = %.1f for 262144 KiB each way -> scale factors %.4f (fetch) and %.4f (write)."
              % (f["copy"], w["copy"], cal_f, cal_w), "",
              "| kernel | FETCH_SIZE avg | WRITE_SIZE avg | scaled read MB | scaled write MB | total MB per launch |", "|---|---|---|---|---|---|"]
    for k in ("ffn_gemm1_kernel", "ffn_gemm2_kernel"):
        d = detail[k]
        lines.append("| %s | %.0f | %.0f | %.1f | %.1f | %.1f |" % (k, f[k], w[k], d["read_bytes"] / 1e6, d["write_bytes"] / 1e6, d["total_bytes"] / 1e6))
    import numpy as np
    import workloads
    cfg = workloads.CONFIGS[workload]
    dest = workloads.config_routing(cfg) // cfg.E_loc
    M = int(np.bincount(dest.ravel(), minlength=cfg.N).max())                  # rows of the hottest receiving rank
    xb, wb_, hb = M * cfg.d * 2, 2 * cfg.E_loc * cfg.d * cfg.f * 2, M * cfg.f * 2
    lines += ["", "Algorithmic bytes of ffn_gemm1_kernel at this workload (M=%d, d=%d, f=%d, %d experts): x %.1f MB + gate/up weights %.1f MB read,"
              % (M, cfg.d, cfg.f, cfg.E_loc, xb / 1e6, wb_ / 1e6),
              "h %.1f MB written = %.1f MB." % (hb / 1e6, (xb + wb_ + hb) / 1e6)]
    lines += ["The fetch counter sits between the L2 and the fabric: it also counts reads served by the 256 MB memory-side cache.",
              "The stored figure (`.json`) carries the SHA-256 of ffn.hip (comments and blank space removed) it was measured on; bench.py reports it as `roofline.traffic` only while that matches.", ""]
    open(base + ".md", "w").write("\n".join(lines))
    print(base + ".md")


def main():
    args = parse()
    if args.summarize_counters:
        summarize_counters(args.workload, *args.summarize_counters)
        return
    if args.gpus != 1:
        print("bench.py measures one GPU only (the library has no multi-GPU path); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import workloads
    import paper_2605_26845_amd as moe

    moe.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = workloads.CONFIGS[args.workload]
    N, E, E_loc, kmax = cfg.N, cfg.E, cfg.E_loc, cfg.kmax
    kb = (N - 1) * (N - 1) + 1                                   # BvN is run uncapped

    # ---------------------------------------------------------------- inputs, resident in HBM
    ids_h = workloads.config_routing(cfg)
    ids = torch.from_numpy(ids_h).to(dev)
    traffic, _ = moe.moe_route_histogram(ids, E)
    torch.cuda.synchronize()
    col = traffic.sum(0).cpu().numpy()
    r = int(np.argmax(col))                                      # hottest receiving rank
    M = int(col[r])
    W = workloads.ffn_weights(E_loc, cfg.d, cfg.f, seed=cfg.seed, dtype=cfg.weight_dtype)
    bf = lambda bits: torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)
    wg, wu, wd = bf(W.w_gate), bf(W.w_up), bf(W.w_down)
    x_h = workloads.activations(M, cfg.d, seed=cfg.seed)
    x = bf(x_h)

    # ---------------------------------------------------------------- preallocated outputs / workspaces
    S = kmax + 2
    traffic = torch.empty((N, N), dtype=torch.int32, device=dev)
    counts = torch.empty((N, E), dtype=torch.int32, device=dev)
    g_out = dict(perms=torch.zeros((1, kmax, N), dtype=torch.uint8, device=dev),
                 durations=torch.zeros((1, kmax), dtype=torch.int32, device=dev),
                 counts=torch.zeros((1,), dtype=torch.int32, device=dev),
                 residual=torch.empty((1, N, N), dtype=torch.int32, device=dev), hashes=None)
    b_out = dict(perms=torch.zeros((1, kb, N), dtype=torch.uint8, device=dev),
                 durations=torch.zeros((1, kb), dtype=torch.int32, device=dev),
                 counts=torch.zeros((1,), dtype=torch.int32, device=dev),
                 residual=torch.empty((1, N, N), dtype=torch.int32, device=dev), hashes=None,
                 pad_total=torch.zeros((1,), dtype=torch.int32, device=dev))
    offsets = torch.empty((S * E_loc + 1,), dtype=torch.int32, device=dev)
    st_ws = torch.empty((moe.load().moe_slice_table_workspace_bytes(N, kmax, E),), dtype=torch.uint8, device=dev)
    ffn_ws = torch.empty((moe.moe_ffn_workspace_bytes(M, cfg.d, cfg.f),), dtype=torch.uint8, device=dev)
    y = torch.empty_like(x)

    main_stream = torch.cuda.current_stream()
    side = torch.cuda.Stream()                                   # default priority
    ev_hist = torch.cuda.Event()
    ev_bvn = torch.cuda.Event()

    def step():
        moe.moe_route_histogram(ids, E, traffic=traffic, expert_counts=counts)
        ev_hist.record(main_stream)
        with torch.cuda.stream(side):
            side.wait_event(ev_hist)
            moe.moe_decompose_bvn(traffic.unsqueeze(0), kb, zero_diag=True, out=b_out)
            ev_bvn.record(side)
        moe.moe_decompose_greedy(traffic.unsqueeze(0), kmax, zero_diag=True, out=g_out)
        moe.moe_slice_table(ids, E, r, traffic, g_out["perms"][0], g_out["durations"][0], g_out["counts"], kmax,
                            offsets=offsets, workspace=st_ws)
        moe.moe_expert_ffn_sliced(x, offsets, S, E_loc, wg, wu, wd, y=y, workspace=ffn_ws)
        main_stream.wait_event(ev_bvn)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.calibration_copy:
        src = torch.ones((256 << 20,), dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)                                           # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    # ---------------------------------------------------------------- timed region
    # HIP events bracket the dominant kernel only: an event pair costs about 7 us of stream time, and with one pair per
    # kernel the step was measured 8 % slower than it is.  The other kernels are timed in a pass of their own below.
    moe.moe_kernel_timing_select("ffn_gemm1_kernel")
    moe.moe_kernel_timing_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    moe.moe_kernel_timing_enable(False)
    kt_dominant = moe.moe_kernel_timing_read()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    assert int(offsets[-1].item()) == M
    # ---------------------------------------------------------------- per-kernel breakdown (not part of the timed region)
    moe.moe_kernel_timing_select(None)
    moe.moe_kernel_timing_enable(True)
    for _ in range(max(5, args.steps // 2)):
        step()
    torch.cuda.synchronize()
    moe.moe_kernel_timing_enable(False)
    kt = moe.moe_kernel_timing_read()
    kt["ffn_gemm1_kernel"] = kt_dominant["ffn_gemm1_kernel"]          # the figure of the timed region

    flops_step = 6.0 * cfg.d * cfg.f * M                         # three GEMMs, 2 flops per MAC
    value = flops_step / (ms_per_step * 1e-3) / 1e12
    kernels = {k: {"avg_us": v[0] * 1e3 / v[1], "launches": v[1]} for k, v in kt.items()}
    g1 = kernels["ffn_gemm1_kernel"]["avg_us"]
    g2 = kernels["ffn_gemm2_kernel"]["avg_us"]
    flops_g1 = 4.0 * cfg.d * cfg.f * M                           # gate and up projections
    achieved = flops_g1 / (g1 * 1e-6) / 1e12
    roofline = {"kernel": "ffn_gemm1_kernel", "bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": stored_traffic(args.workload),
                "avg_launch_us": g1, "flop_per_launch": flops_g1}
    n_match = int(g_out["counts"][0].item())
    n_bvn = int(b_out["counts"][0].item())
    decomp_us = kernels["greedy_kernel"]["avg_us"]
    bvn_us = kernels["bvn_kernel"]["avg_us"]
    result = {
        "metric": "sliced expert-FFN TFLOP/s (% MFMA peak) + decompositions/sec at NxN",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: N=%d ranks, %d experts (%d/rank), top-%d, %d tokens/rank, Zipf s=%.1f; greedy k<=%d vs BvN; "
                               "receiving rank %d (hottest) runs %d SwiGLU experts d=%d ffn=%d on %d rows in %d slices"
                               % (cfg.name, N, E, E_loc, cfg.topk, cfg.T, cfg.zipf_s, kmax, r, E_loc, cfg.d, cfg.f, M, S),
                   "seed": cfg.seed},
        "pct_mfma_peak_whole_step": 100.0 * value / MFMA_BF16_PEAK_TFLOPS,
        "ffn_tflops_kernels_only": flops_step / ((g1 + g2) * 1e-6) / 1e12,
        "decompositions_per_s": {"greedy_%dx%d_k%d" % (N, N, kmax): 1e6 / decomp_us, "bvn_%dx%d_full" % (N, N): 1e6 / bvn_us,
                                 "greedy_matchings": n_match, "bvn_matchings": n_bvn},
        "kernels": kernels,
        "roofline": roofline,
    }

    # ---------------------------------------------------------------- extras outside the timed step
    if not args.no_extras:
        result["extras"] = extras(moe, torch, np, workloads, dev)
        result["extras"].update(ffn_granularity(moe, torch, np, cfg, x, offsets, S, E_loc, wg, wu, wd, y, ffn_ws))
        result["extras"]["makespan_model_us"] = makespan_extras(moe, np, cfg, traffic, g_out, b_out,
                                                                result["extras"]["expert_time_us_vs_rows"])
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, ids_h, r, x_h, W, M)
    print(json.dumps(result))


def stored_traffic(workload):
    """HBM-side bytes per launch of the dominant kernel from the committed counter summary (two rocprofv3 --pmc runs,
    scaled by a plain copy of known size); None if that summary was taken on another workload or if the kernel's
    source has changed since."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "ffn_%s_hbm_traffic.json" % workload)
    try:
        rec = json.load(open(path))
        for rel, digest in rec["source_sha256"].items():
            if code_digest(os.path.join(ROOT, rel)) != digest:
                return None
        return rec["traffic_bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def extras(moe, torch, np, workloads, dev):
    """Batched decomposition (128 x 128 stress matrices) and batched-layer histogram rates."""
    out = {}
    B = 2048
    mats = torch.from_numpy(workloads.stress_matrices(B, 128)).to(dev)
    bufs = dict(perms=torch.zeros((B, 32, 128), dtype=torch.uint8, device=dev),
                durations=torch.zeros((B, 32), dtype=torch.int32, device=dev),
                counts=torch.zeros((B,), dtype=torch.int32, device=dev), residual=None, hashes=None)
    moe.moe_decompose_greedy(mats, 32, zero_diag=True, out=bufs)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    moe.moe_decompose_greedy(mats, 32, zero_diag=True, out=bufs)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    out["greedy_128x128_k32"] = {"matrices": B, "matrices_per_s": B / dt, "matchings_per_s": float(bufs["counts"].sum().item()) / dt}
    # the same batch with the residual held in 16 bits (its entries are below 65536): twice the matrices in flight per CU
    moe.moe_decompose_greedy(mats, 32, zero_diag=True, out=bufs, entries_u16=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    moe.moe_decompose_greedy(mats, 32, zero_diag=True, out=bufs, entries_u16=True)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    out["greedy_128x128_k32_u16"] = {"matrices": B, "matrices_per_s": B / dt, "matchings_per_s": float(bufs["counts"].sum().item()) / dt}
    Bb = 256
    bb = dict(perms=None, durations=None, counts=torch.zeros((Bb,), dtype=torch.int32, device=dev), residual=None,
              hashes=None, pad_total=torch.zeros((Bb,), dtype=torch.int32, device=dev))
    kb = 127 * 127 + 1
    t0 = time.perf_counter()
    moe.moe_decompose_bvn(mats[:Bb], kb, zero_diag=True, out=bb)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    out["bvn_128x128_full"] = {"matrices": Bb, "matrices_per_s": Bb / dt, "matchings_per_s": float(bb["counts"].sum().item()) / dt}
    # the paper's own BvN pipeline (Sinkhorn-Knopp, then BvN in double precision) on dense 8 x 8 traffic (diagonal kept):
    # its evaluation reports up to 50 matchings with many coefficients around 0.03
    B8 = 4096
    m8 = torch.from_numpy(workloads.random_matrices(B8, 8, seed=31, density=1.0, high=2000)).to(dev)
    moe.moe_decompose_sinkhorn_bvn(m8[:8], 50, sweeps=100, want_perms=False, want_scaled=False, want_residual=False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    sk = moe.moe_decompose_sinkhorn_bvn(m8, 50, sweeps=100, want_perms=False, want_scaled=False, want_residual=False)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    cnt = sk["counts"].double()
    coef = sk["coeffs"][sk["coeffs"] > 0]
    out["sinkhorn_bvn_8x8_100_sweeps"] = {"matrices": B8, "matrices_per_s": B8 / dt, "matchings_per_s": float(cnt.sum().item()) / dt,
                                          "mean_matchings": float(cnt.mean().item()), "median_coefficient": float(coef.median().item()),
                                          "max_row_sum_deviation": float(sk["deviation"].max().item())}
    # histogram over 64 layers of the 64-rank top-8 routing shape (16 MiB of ids per layer)
    L, N, T, topk, E = 64, 64, 8192, 8, 256
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    ids = torch.randint(0, E, (L, N, T, topk), dtype=torch.int32, device=dev, generator=g)
    tr = torch.empty((L, N, N), dtype=torch.int32, device=dev)
    cn = torch.empty((L, N, E), dtype=torch.int32, device=dev)
    moe.moe_route_histogram(ids, E, traffic=tr, expert_counts=cn)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    reps = 10
    for _ in range(reps):
        moe.moe_route_histogram(ids, E, traffic=tr, expert_counts=cn)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / reps
    nbytes = ids.numel() * 4 + tr.numel() * 4 + cn.numel() * 4
    out["histogram_64_layers"] = {"bytes": nbytes, "GB_per_s": nbytes / dt / 1e9, "frac_hbm_peak": nbytes / dt / 1e9 / HBM_PEAK_GBS}
    return out


def ffn_granularity(moe, torch, np, cfg, x, offsets, S, E_loc, wg, wu, wd, y, ffn_ws):
    """(i) the same schedule issued as one call per slice (what per-matching launches would cost) beside the single
    call; (ii) expert time against the number of rows of a single slice -- this GPU's version of the paper's Figure 1."""
    out = {}
    dev = x.device
    off_h = offsets.cpu().numpy().astype(np.int64)
    reps = 20

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps * 1e6

    one_call = timed(lambda: moe.moe_expert_ffn_sliced(x, offsets, S, E_loc, wg, wu, wd, y=y, workspace=ffn_ws))
    per_slice = []
    for sl in range(S):
        lo, hi = int(off_h[sl * E_loc]), int(off_h[(sl + 1) * E_loc])
        if hi > lo:
            o = torch.from_numpy((off_h[sl * E_loc:(sl + 1) * E_loc + 1] - lo).astype(np.int32)).to(dev)
            per_slice.append((x[lo:hi], o, y[lo:hi]))

    def run_slices():
        for xs, o, ys in per_slice:
            moe.moe_expert_ffn_sliced(xs, o, 1, E_loc, wg, wu, wd, y=ys, workspace=ffn_ws)

    out["ffn_one_call_us"] = one_call
    # the same call with the dispatch gather / combine scatter fused in: rows in a random arrival order, router weights
    g = torch.Generator(device=dev)
    g.manual_seed(3)
    M_used = int(off_h[-1])
    row_map = torch.randperm(M_used, device=dev, generator=g).to(torch.int32)
    gate = torch.rand((M_used,), device=dev, generator=g)
    out["ffn_one_call_row_map_us"] = timed(lambda: moe.moe_expert_ffn_sliced_mapped(x, offsets, S, E_loc, wg, wu, wd, row_map,
                                                                                    gate, y=y, workspace=ffn_ws))
    out["ffn_one_call_per_slice_us"] = timed(run_slices)
    out["ffn_slices"] = len(per_slice)
    curve = {}
    for rows in (1, 8, 32, 64, 128, 256, 512, 1024, 2048, 4096, 8192):
        if rows > x.shape[0]:
            break
        o = torch.tensor([0, rows] + [rows] * (E_loc - 1), dtype=torch.int32, device=dev)      # all rows on local expert 0
        curve[str(rows)] = timed(lambda: moe.moe_expert_ffn_sliced(x[:rows], o, 1, E_loc, wg, wu, wd, y=y[:rows], workspace=ffn_ws))
    out["expert_time_us_vs_rows"] = curve
    return out


def makespan_extras(moe, np, cfg, traffic, g_out, b_out, curve):
    """Layer completion time of the two schedules under the analytic model of the paper's evaluation, with this GPU's
    measured expert time against rows as the profiling-based cost (and a linear cost through the largest point),
    a circuit of one xGMI link (153 GB/s), bf16 rows of d values, 10 ns reconfiguration."""
    A = traffic.cpu().numpy()
    rows = sorted(int(k) for k in curve)
    table = dict(kind="table", rows=[float(k) for k in rows], seconds=[curve[str(k)] * 1e-6 for k in rows])
    linear = dict(kind="linear", fixed=0.0, per_row=curve[str(rows[-1])] * 1e-6 / rows[-1])
    out = {"assumptions": "153e9 B/s per circuit, %d B per row, 10 ns reconfiguration; residual of the capped schedule "
                          "as one ideal round; profile = expert_time_us_vs_rows" % (2 * cfg.d)}
    for name, o in (("greedy", g_out), ("bvn", b_out)):
        K = int(o["counts"][0].item())
        perms = o["perms"][0, :K].cpu().numpy()
        dur = o["durations"][0, :K].cpu().numpy()
        for mname, model in (("profile", table), ("linear", linear)):
            args = (A, perms, dur, 2.0 * cfg.d, 153e9, 10e-9, model)
            r = moe.moe_makespan_model(*args)
            order = moe.moe_order_matchings(*args)
            ro = moe.moe_makespan_model(*args, order=order)
            out["%s_%s" % (name, mname)] = {"matchings": K, "no_overlap": r["sequential"] * 1e6, "overlap": r["overlap"] * 1e6,
                                            "overlap_johnson_order": ro["overlap"] * 1e6, "ideal_all_to_all": r["ideal"] * 1e6}
    return out


def cpu_baseline(cfg, ids_h, r, x_h, W, M):
    """The CPU oracle, as it stands, on the same workload: integer stages in full, the FFN on a
    bounded sample of rows.  Reported in the metric's unit."""
    import numpy as np
    import oracle
    try:
        from threadpoolctl import threadpool_info
        blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        blas_threads = os.cpu_count() or 1
    t0 = time.perf_counter()
    traffic, _ = oracle.route_histogram(ids_h, cfg.E)
    t_hist = time.perf_counter() - t0
    t0 = time.perf_counter()
    perms, dur, _ = oracle.decompose_greedy(traffic, cfg.kmax, zero_diag=True)
    t_greedy = time.perf_counter() - t0
    t0 = time.perf_counter()
    oracle.decompose_bvn(traffic, None, zero_diag=True)
    t_bvn = time.perf_counter() - t0
    t0 = time.perf_counter()
    offsets, _ = oracle.slice_table(ids_h, cfg.E, r, traffic, perms, dur, cfg.kmax, want_rows=False)
    t_slice = time.perf_counter() - t0
    sample = M                                                   # the whole workload: a few seconds of CPU time
    rows = np.arange(sample)
    t0 = time.perf_counter()
    oracle.expert_ffn_sliced(x_h, offsets, cfg.E_loc, W, rows=rows)
    t_ffn = time.perf_counter() - t0
    tflops = 6.0 * cfg.d * cfg.f * sample / t_ffn / 1e12
    return {"value": tflops, "unit": "TFLOP/s", "cores": int(blas_threads), "kind": "oracle",
            "sample": "FFN: %d of %d rows in float64 numpy (%.2f s, BLAS threads = cores); histogram %.1f ms, greedy %.2f ms, "
                      "BvN %.1f ms, slice table %.1f ms on the full workload, one thread each"
                      % (sample, M, t_ffn, t_hist * 1e3, t_greedy * 1e3, t_bvn * 1e3, t_slice * 1e3),
            "decompositions_per_s": {"greedy": 1.0 / t_greedy, "bvn": 1.0 / t_bvn}}


if __name__ == "__main__":
    main()

#!/usr/bin/env python3
"""Benchmark of the MoE circuit-schedule hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic routing:
    routing histogram -> greedy max-weight decomposition (cap kmax)      [main stream]
                      -> Birkhoff-von Neumann baseline decomposition     [second stream, joined at step end]
                      -> slice table of the receiving rank -> sliced expert SwiGLU FFN
All inputs (router ids, weights, grouped activations) are resident in HBM before the timed
region.  Prints ONE JSON line.  `value` = algorithmic FFN flops of the step / whole step time.

The default workload is the largest bf16 configuration that fits one GPU (c3: one 4096 x 14336
SwiGLU expert, hottest receiving rank).  The other configurations are reported beside it in
`extras` (FFN only for c2 and c4, the batched 128 x 128 decomposition stress workload).
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
SHADER_CLOCK_GHZ = 2.4              # published peak engine clock
VALU_LANES = 256 * 4 * 16           # compute units x SIMDs x lanes: one 32-bit integer operation per lane and cycle
LDS_BYTES_PER_CU = 160 * 1024


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3", choices=["tiny", "c2", "c3", "c4"])
    ap.add_argument("--ffn-kernels", type=int, default=0, choices=[0, 1, 2],
                    help="moe_ffn_tile_override's kernel choice: 0 = the library's own (both phases in one launch where it applies), "
                         "1 = fixed-shape kernels, 2 = adaptive-shape kernels with one launch per phase")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="with --no-extras: still run torch.matmul on the phase-1 shape (so that a profiler run holds the vendor kernel)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 256 MiB device-to-device copy (reference reading for HBM byte counters)")
    ap.add_argument("--summarize-counters", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"),
                    help="no GPU work: turn the counter_collection.csv files of the two rocprofv3 --pmc runs (FETCH_SIZE, "
                         "WRITE_SIZE; both with --calibration-copy) into profiles/ffn_<workload>_hbm_traffic.{md,json}")
    ap.add_argument("--summarize-kernel-stats", metavar="STATS_CSV",
                    help="no GPU work: turn the kernel_stats.csv of a rocprofv3 --kernel-trace --stats run of this script "
                         "into profiles/ffn_<workload>_kernel_stats.md")
    ap.add_argument("--summarize-mfma", metavar="COUNTER_CSV",
                    help="no GPU work: turn the counter_collection.csv of the MFMA-utilisation --pmc run of this script "
                         "into profiles/ffn_<workload>_mfma_utilisation.md")
    return ap.parse_args()


# ------------------------------------------------------------------------------------------------ profile summaries (no GPU)
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


def kernel_key(name):
    """Library kernel behind a profiler kernel name."""
    if "ffn_adaptive_kernel<1" in name or "ffn_gemm_kernel<1," in name:
        return "ffn_gemm1_kernel"
    if "ffn_adaptive_kernel<2" in name or "ffn_gemm_kernel<2," in name:
        return "ffn_gemm2_kernel"
    if "ffn_fused_kernel" in name:
        return "ffn_fused_kernel"
    if "copyBuffer" in name:
        return "copy"
    if name.startswith("Cijk_") or name.startswith("Custom_Cijk_"):
        return "vendor_gemm"
    for k in ("bvn_kernel", "greedy_kernel", "st_count_kernel", "st_scan_kernel", "ffn_plan_kernel", "hist_kernel", "ffn_expand_fp8_kernel"):
        if k in name:
            return k
    return None


FFN_KERNELS = ("ffn_fused_kernel", "ffn_gemm1_kernel", "ffn_gemm2_kernel")


def ffn_kernel_work(cfg, M):
    """Algorithmic flop and bytes per launch of the FFN matrix kernels (phase 1 = gemm1, phase 2 = gemm2, fused = both)."""
    xb, hb = M * cfg.d * 2.0, M * cfg.f * 2.0
    wb = cfg.E_loc * cfg.d * cfg.f * 2.0                                       # one of the three weight matrices, all experts (bf16)
    unit = cfg.d * cfg.f * float(M)
    return {"ffn_gemm1_kernel": {"flop": 4 * unit, "bytes": xb + 2 * wb + hb, "what": "x and gate/up weights read, h written"},
            "ffn_gemm2_kernel": {"flop": 2 * unit, "bytes": hb + wb + xb, "what": "h and down weights read, y written"},
            "ffn_fused_kernel": {"flop": 6 * unit, "bytes": 2 * xb + 3 * wb + 2 * hb, "what": "x and all weights read, h written and read, y written"}}


def profile_suffix(args):
    return "_per_phase" if args.ffn_kernels == 2 else ("_fixed_shape" if args.ffn_kernels == 1 else "")


def bench_flags(args):
    return " --ffn-kernels %d" % args.ffn_kernels if args.ffn_kernels else ""


def workload_shape(workload):
    import numpy as np
    import workloads
    cfg = workloads.CONFIGS[workload]
    dest = workloads.config_routing(cfg) // cfg.E_loc
    M = int(np.bincount(dest.ravel(), minlength=cfg.N).max())                  # rows of the hottest receiving rank
    return cfg, M


def summarize_counters(args, fetch_csv, write_csv):
    """FETCH_SIZE / WRITE_SIZE (KiB per dispatch) of the FFN matrix kernels, scaled by what the same counter reads for the
    256 MiB calibration copy; stored with the SHA-256 of the kernel source it was measured on."""
    import collections
    import csv
    workload = args.workload

    def averages(path):
        acc = collections.defaultdict(list)
        for row in csv.DictReader(open(path)):
            key = kernel_key(row["Kernel_Name"])
            if key:
                acc[key].append(float(row["Counter_Value"]))
        return {k: (max(v) if k == "copy" else sum(v) / len(v)) for k, v in acc.items()}     # the copy: its largest dispatch

    f, w = averages(fetch_csv), averages(write_csv)
    cal_f, cal_w = 262144.0 / f["copy"], 262144.0 / w["copy"]
    cfg, M = workload_shape(workload)
    work = ffn_kernel_work(cfg, M)
    detail = {}
    for k in FFN_KERNELS:
        if k in f and k in w:
            rb, wb = f[k] * cal_f * 1024, w[k] * cal_w * 1024
            detail[k] = {"read_bytes": rb, "write_bytes": wb, "total_bytes": rb + wb, "algorithmic_bytes": work[k]["bytes"],
                         "ratio": (rb + wb) / work[k]["bytes"]}
    rel = "paper_2605_26845_amd/csrc/ffn.hip"
    sha = code_digest(os.path.join(ROOT, rel))
    base = os.path.join(ROOT, "profiles", "ffn_%s%s_hbm_traffic" % (workload, profile_suffix(args)))
    json.dump({"workload": workload, "source_sha256": {rel: sha}, "detail": detail,
               "calibration_factor": {"FETCH_SIZE": cal_f, "WRITE_SIZE": cal_w},
               "see": os.path.basename(base) + ".md"}, open(base + ".json", "w"), indent=1)
    lines = ["# HBM-side byte counters (rocprofv3 --pmc), bench.py workload %s, the FFN matrix kernels" % workload,
             "", "Commands (run from the repository root with TMPDIR=/tmp on the MI355X box, one counter per run; then the summary, no GPU needed):", ""]
    rel_csv = [os.path.relpath(os.path.abspath(c), ROOT) for c in (fetch_csv, write_csv)]      # as given on the command line
    for c, path in zip(("FETCH_SIZE", "WRITE_SIZE"), rel_csv):
        lines.append("    rocprofv3 --pmc %s --output-format csv -d %s -o p -- python3 bench.py --workload %s%s --steps 10 "
                     "--warmup 2 --no-extras --no-cpu-baseline --calibration-copy" % (c, os.path.dirname(path), workload, bench_flags(args)))
    lines += ["    python3 bench.py --workload %s%s --summarize-counters %s %s" % (workload, bench_flags(args), rel_csv[0], rel_csv[1]), "",
              "Calibration: the plain device-to-device copy of 256 MiB (`--calibration-copy`, the largest __amd_rocclr_copyBuffer dispatch) reads",
              "FETCH_SIZE = %.1f and WRITE_SIZE = %.1f for 262144 KiB each way -> scale factors %.4f (fetch) and %.4f (write)."
              % (f["copy"], w["copy"], cal_f, cal_w), "",
              "| kernel | FETCH_SIZE avg | WRITE_SIZE avg | scaled read MB | scaled write MB | total MB per launch | algorithmic MB | ratio |", "|---|---|---|---|---|---|---|---|"]
    for k, d in detail.items():
        lines.append("| %s | %.0f | %.0f | %.1f | %.1f | %.1f | %.1f | %.2f |" % (k, f[k], w[k], d["read_bytes"] / 1e6, d["write_bytes"] / 1e6,
                                                                         d["total_bytes"] / 1e6, d["algorithmic_bytes"] / 1e6, d["ratio"]))
    lines += ["", "Algorithmic bytes at this workload (M=%d rows, d=%d, f=%d, %d experts, bf16):" % (M, cfg.d, cfg.f, cfg.E_loc)]
    lines += ["- %s: %s = %.1f MB" % (k, work[k]["what"], work[k]["bytes"] / 1e6) for k in detail]
    lines += ["The fetch counter sits between a die's L2 and the fabric: it also counts reads served by the 256 MB memory-side cache, and an operand",
              "strip shared by the tiles of two dies is fetched once per die.",
              "The stored figures (`.json`) carry the SHA-256 of ffn.hip (comments and blank space removed) they were measured on; bench.py reports",
              "the dominant kernel's as `roofline.traffic` only while that matches.", ""]
    open(base + ".md", "w").write("\n".join(lines))
    print(base + ".md")


def summarize_kernel_stats(args, stats_csv):
    import csv
    workload = args.workload
    cfg, M = workload_shape(workload)
    work = ffn_kernel_work(cfg, M)
    rel = os.path.relpath(os.path.abspath(stats_csv), ROOT)
    out_dir, prefix = os.path.dirname(rel), os.path.basename(rel).replace("_kernel_stats.csv", "")
    lines = ["# rocprofv3 kernel-trace summary: bench.py, workload %s (N=%d, %d experts, top-%d, %d tokens/rank; %d experts d=%d f=%d; hottest rank: %d rows)"
             % (workload, cfg.N, cfg.E, cfg.topk, cfg.T, cfg.E_loc, cfg.d, cfg.f, M), "",
             "Commands (run from the repository root with TMPDIR=/tmp on the MI355X box; then the summary, no GPU needed):", "",
             "    rocprofv3 --kernel-trace --stats --output-format csv -d %s -o %s -- python3 bench.py --workload %s%s --steps 20 --no-extras --no-cpu-baseline"
             % (out_dir, prefix, workload, bench_flags(args)),
             "    python3 bench.py --workload %s%s --summarize-kernel-stats %s" % (workload, bench_flags(args), rel), "",
             "(library kernels only, times in microseconds; the run also holds bench.py's passes with one event pair per kernel and, unless",
             "--ffn-kernels is given, with one launch per FFN phase: the phase kernels below come from that pass)", "",
             "| kernel | calls | avg us | min us | max us | % of GPU time |", "|---|---|---|---|---|---|"]
    avg = {}
    for row in csv.DictReader(open(stats_csv)):
        key = kernel_key(row["Name"])
        if key is None or key == "copy":
            continue
        name = row["Name"].replace("(anonymous namespace)::", "").replace("void ", "").split("(")[0]
        lines.append("| %s | %s | %.1f | %.1f | %.1f | %s |" % (name, row["Calls"], float(row["AverageNs"]) / 1e3, float(row["MinNs"]) / 1e3,
                                                            float(row["MaxNs"]) / 1e3, row["Percentage"]))
        avg[key] = float(row["AverageNs"]) / 1e3
    lines += ["", "bench.py reports ffn_fused_kernel (both FFN phases in one launch), or the phase-1 kernel (gate / up projections + SwiGLU) as",
              "ffn_gemm1_kernel and the phase-2 kernel (down projection) as ffn_gemm2_kernel; the average of the kernel the bench line names in",
              "`roofline.kernel` must agree with its `roofline.avg_launch_us` (HIP events inside the library; the profiler's own overhead and the",
              "box-to-box spread of about 5 % are the difference)."]
    for k in FFN_KERNELS:
        if k in avg:
            lines.append("- %s: %.4g flop per launch / %.1f us = %.0f TFLOP/s = %.3f of the 2.5 PFLOP/s bf16 MFMA peak"
                         % (k, work[k]["flop"], avg[k], work[k]["flop"] / avg[k] / 1e6, work[k]["flop"] / avg[k] / 1e6 / MFMA_BF16_PEAK_TFLOPS))
    lines.append("")
    path = os.path.join(ROOT, "profiles", "ffn_%s%s_kernel_stats.md" % (workload, profile_suffix(args)))
    open(path, "w").write("\n".join(lines))
    print(path)


MFMA_COUNTERS = ["SQ_VALU_MFMA_BUSY_CYCLES", "SQ_BUSY_CYCLES", "SQ_BUSY_CU_CYCLES", "SQ_WAVE_CYCLES", "SQ_WAIT_ANY", "SQ_LDS_BANK_CONFLICT",
                 "SQ_INSTS_VALU_MFMA_MOPS_BF16", "GRBM_GUI_ACTIVE"]


def summarize_mfma(args, counter_csv):
    """MFMA utilisation of the FFN kernels from one rocprofv3 --pmc run (averages over the dispatches of each kernel)."""
    import collections
    import csv
    workload = args.workload
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    dur = collections.defaultdict(dict)
    for row in csv.DictReader(open(counter_csv)):
        key = kernel_key(row["Kernel_Name"])
        if key in FFN_KERNELS or key == "vendor_gemm":
            acc[key][row["Counter_Name"]].append(float(row["Counter_Value"]))
            dur[key][row["Dispatch_Id"]] = float(row["End_Timestamp"]) - float(row["Start_Timestamp"])
    cfg, M = workload_shape(workload)
    rel = os.path.relpath(os.path.abspath(counter_csv), ROOT)
    lines = ["# MFMA utilisation counters (rocprofv3 --pmc), bench.py workload %s, the FFN matrix kernels" % workload, "",
             "Commands (run from the repository root with TMPDIR=/tmp on the MI355X box; then the summary, no GPU needed):", "",
             "    rocprofv3 --kernel-trace --pmc %s --output-format csv -d %s -o p -- python3 bench.py --workload %s%s --steps 10 --warmup 2 --no-extras --no-cpu-baseline --vendor-gemm"
             % (" ".join(MFMA_COUNTERS), os.path.dirname(rel), workload, bench_flags(args)),
             "    python3 bench.py --workload %s%s --summarize-mfma %s" % (workload, bench_flags(args), rel), "",
             "(the run also holds bench.py's pass with one launch per FFN phase: the phase kernels below come from that pass; vendor_gemm is",
             "torch.matmul on the shape and data of phase 1, x [M][d] times one expert's gate and up weights [2f][d]^T, the same flop as",
             "ffn_gemm1_kernel when the rank holds one expert)", "",
             "Averages per dispatch, as the profiler reports them: SQ_* counters are sums over the chip (SQ_VALU_MFMA_BUSY_CYCLES over its 1024 SIMDs,",
             "SQ_BUSY_CU_CYCLES over its 256 compute units, SQ_WAVE_CYCLES / SQ_WAIT_ANY over all wavefronts), GRBM_GUI_ACTIVE is the sum of the busy",
             "shader-clock cycles of the 8 accelerator dies (so cycles per launch = GRBM_GUI_ACTIVE / 8).", ""]
    names = sorted({c for k in acc for c in acc[k]})
    kernels = [k for k in FFN_KERNELS + ("vendor_gemm",) if k in acc]
    lines += ["| counter | " + " | ".join(kernels) + " |", "|---|" + "---|" * len(kernels)]
    mean = {k: {c: sum(v) / len(v) for c, v in acc[k].items()} for k in kernels}
    for c in names:
        lines.append("| %s | " % c + " | ".join("%.4g" % mean[k].get(c, float("nan")) for k in kernels) + " |")
    lines.append("| dispatches | " + " | ".join("%d" % len(dur[k]) for k in kernels) + " |")
    lines.append("| average duration under the profiler, us | " + " | ".join("%.1f" % (sum(dur[k].values()) / len(dur[k]) / 1e3) for k in kernels) + " |")
    lines.append("")
    flops = {k: v["flop"] for k, v in ffn_kernel_work(cfg, M).items()}
    flops["vendor_gemm"] = 4.0 * cfg.d * cfg.f * M
    peak_per_cycle = MFMA_BF16_PEAK_TFLOPS * 1e12 / (SHADER_CLOCK_GHZ * 1e9)
    for k in kernels:
        m = mean[k]
        us = sum(dur[k].values()) / len(dur[k]) / 1e3
        lines.append("%s:" % k)
        if "GRBM_GUI_ACTIVE" in m:
            cyc = m["GRBM_GUI_ACTIVE"] / 8.0
            lines.append("- shader clock while it ran: %.3g cycles / %.1f us = %.2f GHz (%.1f GHz is the published peak clock the 2.5 PFLOP/s assume);" % (cyc, us, cyc / us / 1e3, SHADER_CLOCK_GHZ))
            lines.append("- %.4g flop per launch / %.3g cycles = %.0f flop per cycle = %.3f of the %.0f flop per cycle of 256 compute units;" % (flops[k], cyc, flops[k] / cyc, flops[k] / cyc / peak_per_cycle, peak_per_cycle))
            if "SQ_VALU_MFMA_BUSY_CYCLES" in m:
                lines.append("- MFMA pipes busy %.1f %% of the launch's cycles (SQ_VALU_MFMA_BUSY_CYCLES / (1024 SIMDs x cycles per launch));" % (100.0 * m["SQ_VALU_MFMA_BUSY_CYCLES"] / (1024.0 * cyc)))
        if "SQ_VALU_MFMA_BUSY_CYCLES" in m and m.get("SQ_BUSY_CU_CYCLES", 0) > 0:
            lines.append("- MFMA pipes busy %.1f %% of the cycles a compute unit had work (SQ_VALU_MFMA_BUSY_CYCLES / (4 x SQ_BUSY_CU_CYCLES));" % (100.0 * m["SQ_VALU_MFMA_BUSY_CYCLES"] / 4.0 / m["SQ_BUSY_CU_CYCLES"]))
        if "SQ_WAIT_ANY" in m and m.get("SQ_WAVE_CYCLES", 0) > 0:
            lines.append("- wavefronts waiting on a memory / LDS counter %.1f %% of their cycles (SQ_WAIT_ANY / SQ_WAVE_CYCLES);" % (100.0 * m["SQ_WAIT_ANY"] / m["SQ_WAVE_CYCLES"]))
        if "SQ_LDS_BANK_CONFLICT" in m and m.get("SQ_BUSY_CU_CYCLES", 0) > 0:
            lines.append("- LDS bank-conflict cycles: %.2f %% of the busy compute-unit cycles." % (100.0 * m["SQ_LDS_BANK_CONFLICT"] / m["SQ_BUSY_CU_CYCLES"]))
        lines.append("")
    path = os.path.join(ROOT, "profiles", "ffn_%s%s_mfma_utilisation.md" % (workload, profile_suffix(args)))
    open(path, "w").write("\n".join(lines))
    print(path)


def stored_traffic(workload, kernel):
    """HBM-side bytes per launch of the dominant kernel from the committed counter summary (two rocprofv3 --pmc runs,
    scaled by a plain copy of known size); None if that summary was taken on another workload or if the kernel's
    source has changed since."""
    path = os.path.join(ROOT, "profiles", "ffn_%s_hbm_traffic.json" % workload)       # (the default kernel choice)
    try:
        rec = json.load(open(path))
        for rel, digest in rec["source_sha256"].items():
            if code_digest(os.path.join(ROOT, rel)) != digest:
                return None
        return rec["detail"][kernel]["total_bytes"]
    except (OSError, KeyError, ValueError):
        return None


# ------------------------------------------------------------------------------------------------ workloads on the device
class Workload:
    """Inputs of one configuration, resident in HBM: router ids, the hottest receiving rank, its expert weights and
    activations, and every output / workspace buffer of the path."""

    def __init__(self, moe, torch, np, workloads, cfg, dev, device_weights=False):
        self.cfg = cfg
        N, E, E_loc, kmax = cfg.N, cfg.E, cfg.E_loc, cfg.kmax
        self.kb = (N - 1) * (N - 1) + 1                               # BvN is run uncapped
        self.ids_h = workloads.config_routing(cfg)
        self.ids = torch.from_numpy(self.ids_h).to(dev)
        traffic, _ = moe.moe_route_histogram(self.ids, E)
        torch.cuda.synchronize()
        col = traffic.sum(0).cpu().numpy()
        self.r = int(np.argmax(col))                                  # hottest receiving rank
        self.M = M = int(col[self.r])
        bf = lambda bits: torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)
        if device_weights:
            self.W = None
            self.w = workloads.ffn_weights_on_device(E_loc, cfg.d, cfg.f, cfg.seed, cfg.weight_dtype, dev)
        else:
            self.W = W = workloads.ffn_weights(E_loc, cfg.d, cfg.f, seed=cfg.seed, dtype=cfg.weight_dtype)
            if W.dtype == "bf16":
                self.w = dict(w_gate=bf(W.w_gate), w_up=bf(W.w_up), w_down=bf(W.w_down))
            else:
                up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
                self.w = dict(w_gate=up(W.w_gate), w_up=up(W.w_up), w_down=up(W.w_down), s_gate=up(W.s_gate), s_up=up(W.s_up), s_down=up(W.s_down))
        self.x = workloads.activations_on_device(M, cfg.d, cfg.seed, dev)
        self.S = S = kmax + 2
        self.traffic = torch.empty((N, N), dtype=torch.int32, device=dev)
        self.counts = torch.empty((N, E), dtype=torch.int32, device=dev)
        self.g_out = dict(perms=torch.zeros((1, kmax, N), dtype=torch.uint8, device=dev),
                          durations=torch.zeros((1, kmax), dtype=torch.int32, device=dev),
                          counts=torch.zeros((1,), dtype=torch.int32, device=dev),
                          residual=torch.empty((1, N, N), dtype=torch.int32, device=dev), hashes=None)
        self.b_out = dict(perms=torch.zeros((1, self.kb, N), dtype=torch.uint8, device=dev),
                          durations=torch.zeros((1, self.kb), dtype=torch.int32, device=dev),
                          counts=torch.zeros((1,), dtype=torch.int32, device=dev),
                          residual=torch.empty((1, N, N), dtype=torch.int32, device=dev), hashes=None,
                          pad_total=torch.zeros((1,), dtype=torch.int32, device=dev))
        self.offsets = torch.empty((S * E_loc + 1,), dtype=torch.int32, device=dev)
        self.st_ws = torch.empty((moe.load().moe_slice_table_workspace_bytes(N, kmax, E),), dtype=torch.uint8, device=dev)
        ws = moe.moe_ffn_workspace_bytes(M, cfg.d, cfg.f)
        if cfg.weight_dtype == "fp8":
            ws += moe.moe_ffn_expanded_weights_bytes(E_loc, cfg.d, cfg.f)
        self.ffn_ws = torch.empty((ws,), dtype=torch.uint8, device=dev)
        self.y = torch.empty_like(self.x)
        self.moe, self.torch = moe, torch
        self.main_stream = torch.cuda.current_stream()
        self.side = torch.cuda.Stream()                               # default priority
        self.ev_hist = torch.cuda.Event()
        self.ev_bvn = torch.cuda.Event()

    def describe(self):
        c = self.cfg
        return ("%s: N=%d ranks, %d experts (%d/rank), top-%d, %d tokens/rank, Zipf s=%.1f; greedy k<=%d vs BvN; receiving rank %d "
                "(hottest) runs %d SwiGLU experts d=%d ffn=%d (%s weights) on %d rows in %d slices"
                % (c.name, c.N, c.E, c.E_loc, c.topk, c.T, c.zipf_s, c.kmax, self.r, c.E_loc, c.d, c.f, c.weight_dtype, self.M, self.S))

    def ffn(self):
        self.moe.moe_expert_ffn_sliced(self.x, self.offsets, self.S, self.cfg.E_loc, y=self.y, workspace=self.ffn_ws, **self.w)

    def step(self):
        moe, torch, c = self.moe, self.torch, self.cfg
        moe.moe_route_histogram(self.ids, c.E, traffic=self.traffic, expert_counts=self.counts)
        self.ev_hist.record(self.main_stream)
        with torch.cuda.stream(self.side):
            self.side.wait_event(self.ev_hist)
            moe.moe_decompose_bvn(self.traffic.unsqueeze(0), self.kb, zero_diag=True, out=self.b_out)
            self.ev_bvn.record(self.side)
        moe.moe_decompose_greedy(self.traffic.unsqueeze(0), c.kmax, zero_diag=True, out=self.g_out)
        moe.moe_slice_table(self.ids, c.E, self.r, self.traffic, self.g_out["perms"][0], self.g_out["durations"][0],
                            self.g_out["counts"], c.kmax, offsets=self.offsets, workspace=self.st_ws)
        self.ffn()
        self.main_stream.wait_event(self.ev_bvn)


def kernel_times(moe, torch, fn, reps):
    """Average duration per kernel name (us) over `reps` calls of fn, from HIP events around every kernel, and the wall
    time per call (s)."""
    for _ in range(2):
        fn()
    torch.cuda.synchronize()
    moe.moe_kernel_timing_select(None)
    moe.moe_kernel_timing_enable(True)
    t0 = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / reps
    moe.moe_kernel_timing_enable(False)
    kt = moe.moe_kernel_timing_read()
    return {k: v[0] * 1e3 / v[1] for k, v in kt.items()}, dt


def ffn_kernel_us(times):
    """(matrix kernels, the other FFN kernels) of one call, us."""
    gemm = sum(v for k, v in times.items() if k in ("ffn_fused_kernel", "ffn_gemm1_kernel", "ffn_gemm2_kernel"))
    other = sum(v for k, v in times.items() if k in ("ffn_plan_kernel", "ffn_expand_fp8_kernel"))
    return gemm, other


def graph_replay_step(moe, torch, wl, reps):
    """The whole step recorded once into a HIP graph (the library makes no runtime call but kernel launches, so the
    capture holds the histogram, both decompositions -- BvN on a forked branch --, the slice table and the FFN) and
    replayed: what the launches and the gaps between them cost the eager step.  Wall time per replay; errors are reported,
    not raised (a measurement beside the headline, not part of it)."""
    c = wl.cfg
    try:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            cur = torch.cuda.current_stream()
            moe.moe_route_histogram(wl.ids, c.E, traffic=wl.traffic, expert_counts=wl.counts)
            wl.side.wait_stream(cur)
            with torch.cuda.stream(wl.side):
                moe.moe_decompose_bvn(wl.traffic.unsqueeze(0), wl.kb, zero_diag=True, out=wl.b_out)
            moe.moe_decompose_greedy(wl.traffic.unsqueeze(0), c.kmax, zero_diag=True, out=wl.g_out)
            moe.moe_slice_table(wl.ids, c.E, wl.r, wl.traffic, wl.g_out["perms"][0], wl.g_out["durations"][0],
                                wl.g_out["counts"], c.kmax, offsets=wl.offsets, workspace=wl.st_ws)
            wl.ffn()
            cur.wait_stream(wl.side)
        for _ in range(2):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) / reps * 1e6
        wl.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            wl.step()
        torch.cuda.synchronize()
        eager_us = (time.perf_counter() - t0) / reps * 1e6
        return {"replay_us": us, "eager_us": eager_us, "tflops_replay": 6.0 * c.d * c.f * wl.M / us / 1e6}
    except Exception as exc:                                              # noqa: BLE001
        torch.cuda.synchronize()
        return {"error": str(exc)[:200]}


def ffn_entry(moe, torch, wl, reps, kernels):
    """FFN figures of one workload: inside the whole step (the decompositions run before and beside the FFN, as in the
    timed region), with the FFN call issued back to back (the chip then never idles between two calls and settles at a
    lower clock under its power limit), and with one launch per phase (moe_ffn_tile_override) for the figures per phase."""
    cfg, M = wl.cfg, wl.M
    step_us, step_s = kernel_times(moe, torch, wl.step, reps)
    e = ffn_figures(cfg, M, wl.S, *ffn_kernel_us(step_us))
    e["step_kernels_us"] = step_us
    e["step_ms_with_an_event_pair_per_kernel"] = step_s * 1e3
    b2b, _ = kernel_times(moe, torch, wl.ffn, reps)
    g, _ = ffn_kernel_us(b2b)
    e["back_to_back"] = {"matrix_kernels_us": g, "frac_mfma_peak": 6.0 * cfg.d * cfg.f * M / g / 1e6 / MFMA_BF16_PEAK_TFLOPS}
    moe.moe_ffn_tile_override(0, 2 if kernels == 0 else kernels, 0)
    try:
        ph, _ = kernel_times(moe, torch, wl.step, reps)
    finally:
        moe.moe_ffn_tile_override(0, kernels, 0)
    e["one_launch_per_phase"] = phase_figures(cfg, M, ph["ffn_gemm1_kernel"], ph["ffn_gemm2_kernel"])
    return e


def backward_entry(moe, torch, workloads, wl, reps):
    """The backward pass of the same schedule (second workload: dx and the three weight gradients per expert; bf16 weights
    only): time per call and per kernel; algorithmic flop = 12*d*f*M (dh 2, dx 4, weight gradients 6), executed 16*d*f*M
    (the gate / up projections are recomputed)."""
    cfg, M = wl.cfg, wl.M
    if cfg.weight_dtype != "bf16":
        return None
    dy = workloads.activations_on_device(M, cfg.d, cfg.seed + 9, wl.x.device)
    ws = torch.empty((int(moe.load().moe_ffn_backward_workspace_bytes(M, cfg.E_loc, cfg.d, cfg.f)),), dtype=torch.uint8, device=wl.x.device)
    fn = lambda: moe.moe_expert_ffn_backward_sliced(wl.x, dy, wl.offsets, wl.S, cfg.E_loc, wl.w["w_gate"], wl.w["w_up"], wl.w["w_down"], workspace=ws)
    times, dt = kernel_times(moe, torch, fn, reps)
    gemm = sum(v for k, v in times.items() if k.startswith("ffn_bwd_"))
    alg = 12.0 * cfg.d * cfg.f * M
    return {"rows": M, "call_us": dt * 1e6, "tflops_algorithmic": alg / dt / 1e12, "frac_mfma_peak_algorithmic": alg / dt / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "matrix_kernels_us": gemm, "tflops_executed_in_matrix_kernels": 16.0 * cfg.d * cfg.f * M / gemm / 1e6,
            "workspace_GB": ws.numel() / 1e9, "kernels_us": times}


def phase_figures(cfg, M, g1_us, g2_us):
    f1, f2 = 4.0 * cfg.d * cfg.f * M, 2.0 * cfg.d * cfg.f * M
    return {"phase1_us": g1_us, "phase2_us": g2_us, "phase1_tflops": f1 / g1_us / 1e6, "phase2_tflops": f2 / g2_us / 1e6,
            "phase1_frac_mfma_peak": f1 / g1_us / 1e6 / MFMA_BF16_PEAK_TFLOPS, "phase2_frac_mfma_peak": f2 / g2_us / 1e6 / MFMA_BF16_PEAK_TFLOPS,
            "frac_mfma_peak_both": (f1 + f2) / (g1_us + g2_us) / 1e6 / MFMA_BF16_PEAK_TFLOPS}


def ffn_figures(cfg, M, S, gemm_us, other_us):
    flops = 6.0 * cfg.d * cfg.f * M
    wbytes = (1 if cfg.weight_dtype == "fp8" else 2) * 3.0 * cfg.d * cfg.f * cfg.E_loc
    abytes = 4.0 * cfg.d * M + 4.0 * cfg.f * M + wbytes                 # x in, y out, h written and read, weights once
    intensity = flops / abytes
    ridge = MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    return {"rows": M, "slices": S, "experts": cfg.E_loc, "d": cfg.d, "f": cfg.f, "weights": cfg.weight_dtype,
            "matrix_kernels_us": gemm_us, "plan_and_other_kernels_us": other_us,
            "ffn_tflops_kernels_only": flops / gemm_us / 1e6, "frac_mfma_peak_kernels_only": flops / gemm_us / 1e6 / MFMA_BF16_PEAK_TFLOPS,
            "algorithmic_flop_per_byte": intensity, "bound": "mfma" if intensity > ridge else "hbm",
            "note": "bf16 MFMA peak is the denominator for fp8 weights too: they are dequantised to bf16 on the way to the matrix cores"}


def main():
    args = parse()
    if args.summarize_counters:
        summarize_counters(args, *args.summarize_counters)
        return
    if args.summarize_kernel_stats:
        summarize_kernel_stats(args, args.summarize_kernel_stats)
        return
    if args.summarize_mfma:
        summarize_mfma(args, args.summarize_mfma)
        return
    if args.gpus != 1:
        print("bench.py measures one GPU only (the library has no multi-GPU path); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import workloads
    import paper_2605_26845_amd as moe

    moe.load()
    moe.moe_ffn_tile_override(0, args.ffn_kernels, 0)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = workloads.CONFIGS[args.workload]
    wl = Workload(moe, torch, np, workloads, cfg, dev)
    M, N, kmax = wl.M, cfg.N, cfg.kmax

    for _ in range(args.warmup):
        wl.step()
    torch.cuda.synchronize()
    if args.calibration_copy:
        src = torch.ones((256 << 20,), dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)                                           # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    # ---------------------------------------------------------------- timed region
    # HIP events bracket the dominant kernel only: an event pair costs about 7 us of stream time, and with one pair per
    # kernel a step of small kernels is measured slower than it is.  The other kernels are timed in a pass of their own.
    names, _ = kernel_times(moe, torch, wl.step, 1)
    dominant = "ffn_fused_kernel" if "ffn_fused_kernel" in names else "ffn_gemm1_kernel"
    moe.moe_kernel_timing_select(dominant)
    moe.moe_kernel_timing_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        wl.step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    moe.moe_kernel_timing_enable(False)
    kt_dominant = moe.moe_kernel_timing_read()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    assert int(wl.offsets[-1].item()) == M
    # ---------------------------------------------------------------- per-kernel breakdown (not part of the timed region)
    step_us, _ = kernel_times(moe, torch, wl.step, max(5, args.steps // 2))
    kernels = {k: {"avg_us": v} for k, v in step_us.items()}
    kernels[dominant] = {"avg_us": kt_dominant[dominant][0] * 1e3 / kt_dominant[dominant][1], "launches": kt_dominant[dominant][1],
                         "note": "the figure of the timed region"}
    # one launch per phase, for the figures per phase (the default issues both phases in one launch where it applies)
    moe.moe_ffn_tile_override(0, 2 if args.ffn_kernels == 0 else args.ffn_kernels, 0)
    ph_us, _ = kernel_times(moe, torch, wl.step, max(5, args.steps // 2))
    moe.moe_ffn_tile_override(0, args.ffn_kernels, 0)

    flops_step = 6.0 * cfg.d * cfg.f * M                         # three GEMMs, 2 flops per MAC
    value = flops_step / (ms_per_step * 1e-3) / 1e12
    dom_us = kernels[dominant]["avg_us"]
    flops_dom = flops_step if dominant == "ffn_fused_kernel" else 4.0 * cfg.d * cfg.f * M
    achieved = flops_dom / (dom_us * 1e-6) / 1e12
    roofline = {"kernel": dominant, "bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": stored_traffic(args.workload, dominant),
                "avg_launch_us": dom_us, "flop_per_launch": flops_dom,
                "what": "both FFN phases in one launch: 6*d*f*M flop" if dominant == "ffn_fused_kernel" else "phase 1 (gate / up + SwiGLU): 4*d*f*M flop"}
    n_match = int(wl.g_out["counts"][0].item())
    n_bvn = int(wl.b_out["counts"][0].item())
    decomp_us = kernels["greedy_kernel"]["avg_us"]
    bvn_us = kernels["bvn_kernel"]["avg_us"]
    gemm_us, other_us = ffn_kernel_us({k: v["avg_us"] for k, v in kernels.items()})
    result = {
        "metric": "sliced expert-FFN TFLOP/s (% MFMA peak) + decompositions/sec at NxN",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.describe(), "seed": cfg.seed},
        "pct_mfma_peak_whole_step": 100.0 * value / MFMA_BF16_PEAK_TFLOPS,
        "ffn_tflops_kernels_only": flops_step / (gemm_us * 1e-6) / 1e12,
        "ffn_one_launch_per_phase": phase_figures(cfg, M, ph_us["ffn_gemm1_kernel"], ph_us["ffn_gemm2_kernel"]),
        "decompositions_per_s": {"greedy_%dx%d_k%d" % (N, N, kmax): 1e6 / decomp_us, "bvn_%dx%d_full" % (N, N): 1e6 / bvn_us,
                                 "greedy_matchings": n_match, "bvn_matchings": n_bvn},
        "kernels": kernels,
        "roofline": roofline,
    }

    # ---------------------------------------------------------------- extras outside the timed step
    if not args.no_extras:
        ex = result["extras"] = {}
        ex["ffn_by_config"] = {cfg.name: ffn_figures(cfg, M, wl.S, gemm_us, other_us)}
        ex["ffn_by_config"][cfg.name]["one_launch_per_phase"] = result["ffn_one_launch_per_phase"]
        ex["vendor_gemm_same_shape"] = vendor_gemm(torch, wl)
        ex["step_as_hip_graph"] = {cfg.name: graph_replay_step(moe, torch, wl, 10)}
        ex["mfma_only_probe"] = mfma_probe(moe, torch)
        roofline["measured_mfma_only_tflops"] = ex["mfma_only_probe"]["ffn_like_operands"]["tflops"]
        ex["backward_by_config"] = {cfg.name: backward_entry(moe, torch, workloads, wl, 3)}
        ex.update(ffn_granularity(moe, torch, np, wl))
        ex["makespan_model_us"] = makespan_extras(moe, np, cfg, wl.traffic, wl.g_out, wl.b_out, ex["expert_time_us_vs_rows"])
        x_sample, sample_rows = None, None
        if not args.no_cpu_baseline:
            sample_rows = np.unique(np.linspace(0, M - 1, num=min(M, cpu_sample_rows(cfg)), dtype=np.int64))
            x_sample = wl.x[torch.from_numpy(sample_rows).to(dev)].view(torch.int16).cpu().numpy().view(np.uint16)
        offsets_h = wl.offsets.cpu().numpy()
        ids_h, r_main, W_main = wl.ids_h, wl.r, wl.W
        del wl
        torch.cuda.empty_cache()
        for name in ("c2", "c3", "c4"):
            if name == cfg.name:
                continue
            other_wl = Workload(moe, torch, np, workloads, workloads.CONFIGS[name], dev, device_weights=(name == "c4"))
            ex["ffn_by_config"][name] = ffn_entry(moe, torch, other_wl, 10 if name == "c2" else 3, args.ffn_kernels)
            ex["ffn_by_config"][name]["workload"] = other_wl.describe()
            if name == "c2":
                ex["step_as_hip_graph"][name] = graph_replay_step(moe, torch, other_wl, 30)
            bw = backward_entry(moe, torch, workloads, other_wl, 10 if name == "c2" else 3)
            if bw is not None:
                ex["backward_by_config"][name] = bw
            del other_wl
            torch.cuda.empty_cache()
        ex.update(decomposition_extras(moe, torch, np, workloads, dev, cpu=not args.no_cpu_baseline))
        ex.update(histogram_and_sinkhorn_extras(moe, torch, np, workloads, dev))
        ex["popularity_jitter_16_ranks"] = jitter_extras(moe, torch, np, workloads, dev)
        ex["fragmentation_16_ranks"] = fragmentation_extras(moe, torch, np, workloads, dev)
        if not args.no_cpu_baseline:
            result["cpu_baseline"] = cpu_baseline(cfg, ids_h, r_main, x_sample, sample_rows, offsets_h, W_main, M)
            result["cpu_baseline"]["decomposition_stress"] = ex["decomposition_stress_128x128"].pop("cpu_oracle")
    elif args.vendor_gemm:
        result["vendor_gemm_same_shape"] = vendor_gemm(torch, wl)
    if args.no_extras and not args.no_cpu_baseline:
        sample_rows = np.unique(np.linspace(0, M - 1, num=min(M, cpu_sample_rows(cfg)), dtype=np.int64))
        x_sample = wl.x[torch.from_numpy(sample_rows).to(dev)].view(torch.int16).cpu().numpy().view(np.uint16)
        result["cpu_baseline"] = cpu_baseline(cfg, wl.ids_h, wl.r, x_sample, sample_rows, wl.offsets.cpu().numpy(), wl.W, M)
    print(json.dumps(result))


def cpu_sample_rows(cfg):
    """Rows of the FFN the CPU oracle evaluates: about 1.6e13 float64 flop (10 - 30 s on the host cores of a GPU machine,
    whose BLAS sustains 0.5 - 1.5 TFLOP/s in float64)."""
    return max(256, int(1.6e13 / (6.0 * cfg.d * cfg.f)))


def vendor_gemm(torch, wl):
    """torch.matmul (the vendor GEMM library) on the shape and data of phase 1: x [M][d] times the gate and up weights of
    one expert [2f][d]^T.  Context for `roofline.frac`: what a dense, unsliced bf16 GEMM reaches on this data under the
    same power and clock limits."""
    if wl.cfg.weight_dtype != "bf16":
        return None
    w = torch.cat([wl.w["w_gate"][0], wl.w["w_up"][0]], dim=0)            # [2f][d]
    out = torch.empty((wl.M, w.shape[0]), dtype=torch.bfloat16, device=wl.x.device)
    for _ in range(2):
        torch.matmul(wl.x, w.t(), out=out)
    torch.cuda.synchronize()
    reps = 5
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        torch.matmul(wl.x, w.t(), out=out)
    b.record()
    torch.cuda.synchronize()
    us = a.elapsed_time(b) * 1e3 / reps
    flops = 2.0 * wl.M * w.shape[0] * wl.cfg.d
    return {"shape": "[%d x %d] x [%d x %d]^T, bf16" % (wl.M, wl.cfg.d, w.shape[0], wl.cfg.d), "us": us, "tflops": flops / us / 1e6,
            "frac_mfma_peak": flops / us / 1e6 / MFMA_BF16_PEAK_TFLOPS}


def mfma_probe(moe, torch):
    """The FFN's MFMA instruction issued from registers alone on every SIMD of the chip (no operand moves): the rate
    the matrix cores sustain at the clock the power limit allows, on operands drawn like the FFN's and on zeros."""
    out = {}
    wgs, iters = 256, 100000
    sink = torch.empty((wgs * 256,), dtype=torch.float32, device="cuda")
    flop = wgs * 4.0 * iters * 16 * 32768
    for key, data in (("ffn_like_operands", 1), ("zero_operands", 0)):
        moe.moe_probe_mfma_bf16(data, iters // 10, wgs, sink)
        times, _ = kernel_times(moe, torch, lambda: moe.moe_probe_mfma_bf16(data, iters, wgs, sink), 2)
        us = times["mfma_probe_kernel"]
        out[key] = {"us": us, "tflops": flop / us / 1e6, "frac_mfma_peak": flop / us / 1e6 / MFMA_BF16_PEAK_TFLOPS}
    out["what"] = "v_mfma_f32_32x32x16_bf16 from registers, 4 wavefronts on each of 256 compute units, %d instructions per wavefront" % (16 * iters)
    return out


def decomposition_extras(moe, torch, np, workloads, dev, cpu=True):
    """The batched decomposition stress workload: 8192 independent 128 x 128 matrices, greedy k <= 32 (32-bit residual
    on chip, and the default: 16 bits with a second launch for matrices that do not fit), full BvN on a stated subset,
    with the two bounds that apply (integer ALU throughput; the dependent chain of one wavefront) and the CPU oracle."""
    out = {}
    B, N, K = 8192, 128, 32
    mats_h = workloads.stress_matrices(B, N)
    mats = torch.from_numpy(mats_h).to(dev)
    bufs = dict(perms=torch.zeros((B, K, N), dtype=torch.uint8, device=dev), durations=torch.zeros((B, K), dtype=torch.int32, device=dev),
                counts=torch.zeros((B,), dtype=torch.int32, device=dev), residual=None, hashes=None)
    prof = torch.zeros((B, 4), dtype=torch.int64, device=dev)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    entry = {"matrices": B, "n": N, "kmax": K}
    for label, bits in (("residual_32_bit", 32), ("default_16_bit_with_fallback", 0)):
        dt = timed(lambda: moe.moe_decompose_greedy(mats, K, zero_diag=True, out=bufs, residual_bits=bits))
        matchings = float(bufs["counts"].sum().item())
        # counters of the same launch shape: shader clock the kernel ran at, steps of the augmenting-path searches
        moe.moe_decompose_profile(prof)
        moe.moe_decompose_greedy(mats, K, zero_diag=True, out=bufs, residual_bits=bits)
        torch.cuda.synchronize()
        moe.moe_decompose_profile(None)
        p = prof.cpu().numpy().astype(np.float64)
        clock_ghz = float((p[:, 0] / np.maximum(p[:, 1], 1.0)).mean() * 0.1)          # cycles per 10 ns tick
        steps = float(p[:, 2].mean())
        lds = N * N * (4 if bits == 32 else 2)
        per_cu = min(LDS_BYTES_PER_CU // lds, 32)
        # ALU bound: every step of a search relaxes one row of the residual, N columns at about 6 vector integer
        # operations each (load, add, subtract, compare, two selects) plus the 6-stage minimum reduction; all lanes of
        # the chip at the published clock
        ops_per_matrix = steps * (N * 6.0 + 64 * 6.0)
        alu_bound = VALU_LANES * SHADER_CLOCK_GHZ * 1e9 / ops_per_matrix
        e = {"matrices_per_s": B / dt, "matchings_per_s": matchings / dt, "seconds": dt,
             "lds_limited_wavefronts_per_cu": int(per_cu), "measured_shader_clock_ghz": clock_ghz,
             "search_steps_per_matrix": steps, "searches_per_matrix": float(p[:, 3].mean()),
             "cycles_per_matrix_in_batch": float(p[:, 0].mean()),
             "alu_bound_matrices_per_s": alu_bound, "frac_alu_bound": B / dt / alu_bound,
             "alu_bound_upper_work_k_n3_matrices_per_s": VALU_LANES * SHADER_CLOCK_GHZ * 1e9 / (K * float(N) ** 3 * 6.0)}
        entry[label] = e
    # dependency-chain bound: one wavefront alone on a compute unit is as fast as the chain of dependent steps allows;
    # with w wavefronts resident per compute unit the chip cannot do better than 256 * w times that
    few = 64
    moe.moe_decompose_profile(prof)
    moe.moe_decompose_greedy(mats[:few], K, zero_diag=True, out={k: (v[:few] if v is not None else None) for k, v in bufs.items()}, residual_bits=32)
    torch.cuda.synchronize()
    moe.moe_decompose_profile(None)
    p = prof[:few].cpu().numpy().astype(np.float64)
    alone_s = float((p[:, 1] * 1e-8).mean())                                     # 100 MHz ticks
    alone_clock = float((p[:, 0] / np.maximum(p[:, 1], 1.0)).mean() * 0.1)
    entry["one_wavefront_alone"] = {"seconds_per_matrix": alone_s, "shader_clock_ghz": alone_clock,
                                    "cycles_per_search_step": float((p[:, 0] / np.maximum(p[:, 2], 1.0)).mean())}
    for label in ("residual_32_bit", "default_16_bit_with_fallback"):
        e = entry[label]
        e["chain_bound_matrices_per_s"] = 256 * e["lds_limited_wavefronts_per_cu"] / alone_s
        e["frac_chain_bound"] = e["matrices_per_s"] / e["chain_bound_matrices_per_s"]
    # full Birkhoff-von Neumann (uncapped: up to 16 130 matchings per matrix) on a subset, after a warm-up call
    Bb = 512
    kb = (N - 1) * (N - 1) + 1
    bb = dict(perms=None, durations=None, counts=torch.zeros((Bb,), dtype=torch.int32, device=dev), residual=None,
              hashes=None, pad_total=torch.zeros((Bb,), dtype=torch.int32, device=dev))
    dt = timed(lambda: moe.moe_decompose_bvn(mats[:Bb], kb, zero_diag=True, out=bb))
    entry["bvn_full"] = {"matrices": Bb, "of": B, "matrices_per_s": Bb / dt, "matchings_per_s": float(bb["counts"].sum().item()) / dt,
                         "mean_matchings": float(bb["counts"].double().mean().item()), "seconds": dt,
                         "lds_limited_wavefronts_per_cu": int(LDS_BYTES_PER_CU // (N * N * 4))}
    if cpu:
        import oracle
        threads = min(16, os.cpu_count() or 1)
        ng, nb = 8 * threads, threads
        t0 = time.perf_counter()
        oracle.decompose_batch("greedy", mats_h[:ng], K, zero_diag=True, nthreads=threads, want_perms=False, want_residual=False)
        tg = time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.decompose_batch("bvn", mats_h[:nb], kb, zero_diag=True, nthreads=threads, want_perms=False, want_residual=False)
        tb = time.perf_counter() - t0
        entry["cpu_oracle"] = {"threads": threads, "greedy_k32": {"matrices": ng, "matrices_per_s": ng / tg, "seconds": tg},
                               "bvn_full": {"matrices": nb, "matrices_per_s": nb / tb, "seconds": tb},
                               "sample": "first %d (greedy) / %d (BvN) of the %d stress matrices, OpenMP over matrices" % (ng, nb, B)}
    out["decomposition_stress_128x128"] = entry
    return out


def fragmentation_extras(moe, torch, np, workloads, dev):
    """The paper's point about fragmentation, measured on real kernels (Sections 3.1, 5): the 16-rank configuration's FFN
    on the hottest rank under the greedy schedule (8 matchings + rest: 10 slices), under the full BvN schedule (224
    matchings: 226 slices of a few dozen rows per expert) and unsliced (all rows of an expert in one group)."""
    cfg = workloads.CONFIGS["c2"]
    wl = Workload(moe, torch, np, workloads, cfg, dev)
    wl.step()
    torch.cuda.synchronize()
    out = {}

    def timed(fn, reps=20):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps * 1e6

    out["greedy_schedule"] = {"slices": wl.S, "ffn_us": timed(wl.ffn)}
    kb = wl.kb
    off_b = moe.moe_slice_table(wl.ids, cfg.E, wl.r, wl.traffic, wl.b_out["perms"][0], wl.b_out["durations"][0], wl.b_out["counts"], kb)
    torch.cuda.synchronize()
    assert int(off_b[-1].item()) == wl.M
    sizes = (off_b[1:] - off_b[:-1]).float()
    out["bvn_schedule"] = {"slices": kb + 2, "matchings": int(wl.b_out["counts"][0].item()),
                           "mean_rows_per_nonempty_group": float(sizes[sizes > 0].mean().item()),
                           "ffn_us": timed(lambda: moe.moe_expert_ffn_sliced(wl.x, off_b, kb + 2, cfg.E_loc, y=wl.y, workspace=wl.ffn_ws, **wl.w))}
    # unsliced: the same rows regrouped by expert only (what an all-to-all that delivers everything at once would hand over)
    off_g = wl.offsets.cpu().numpy().astype(np.int64)
    per_expert = np.zeros(cfg.E_loc, dtype=np.int64)
    for g in range(len(off_g) - 1):
        per_expert[g % cfg.E_loc] += off_g[g + 1] - off_g[g]
    off_u = torch.from_numpy(np.concatenate([[0], np.cumsum(per_expert)]).astype(np.int32)).to(dev)
    out["unsliced"] = {"slices": 1, "ffn_us": timed(lambda: moe.moe_expert_ffn_sliced(wl.x, off_u, 1, cfg.E_loc, y=wl.y, workspace=wl.ffn_ws, **wl.w))}
    for k in out:
        out[k]["tflops"] = 6.0 * cfg.d * cfg.f * wl.M / out[k]["ffn_us"] / 1e6
    return out


def jitter_extras(moe, torch, np, workloads, dev):
    """The 16-rank configuration with per-source popularity jitter (every source rank multiplies the expert popularity
    by its own lognormal(0, 0.5) factors): with one popularity for all sources every matching carries about 1/N of the
    traffic; with jitter the matchings are as unequal as in the paper's Figure 2."""
    cfg = workloads.CONFIGS["c2"]
    out = {}
    for label, jit in (("shared_popularity", 0.0), ("per_source_jitter_0.5", 0.5)):
        ids = torch.from_numpy(workloads.config_routing(cfg, per_rank_jitter=jit)).to(dev)
        traffic, _ = moe.moe_route_histogram(ids, cfg.E)
        g = moe.moe_decompose_greedy(traffic.unsqueeze(0), cfg.N * 2, zero_diag=True)
        b = moe.moe_decompose_bvn(traffic.unsqueeze(0), (cfg.N - 1) ** 2 + 1, zero_diag=True)
        torch.cuda.synchronize()
        k = int(g["counts"][0].item())
        A = traffic.clone()
        A.fill_diagonal_(0)
        dur = g["durations"][0, :k].cpu().numpy().astype(float)
        shipped = float(A.sum().item() - g["residual"][0].sum().item())
        out[label] = {"greedy_matchings_uncapped": k, "greedy_durations": [int(v) for v in dur],
                      "greedy_first_%d_ship_fraction" % cfg.kmax: None, "bvn_matchings": int(b["counts"][0].item()),
                      "ideal_all_to_all_rows": int(b["pad_total"][0].item()), "sum_of_greedy_durations": int(dur.sum()),
                      "off_diagonal_rows": int(A.sum().item()), "shipped_uncapped": shipped}
        gk = moe.moe_decompose_greedy(traffic.unsqueeze(0), cfg.kmax, zero_diag=True)
        torch.cuda.synchronize()
        out[label]["greedy_first_%d_ship_fraction" % cfg.kmax] = 1.0 - float(gk["residual"][0].sum().item()) / float(A.sum().item())
    return out


def histogram_and_sinkhorn_extras(moe, torch, np, workloads, dev):
    out = {}
    # the paper's own BvN pipeline (Sinkhorn-Knopp, then BvN in double precision) on dense 8 x 8 traffic (diagonal kept):
    # Section 5 describes decompositions of about 50 matchings whose coefficients are a few hundredths
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
    del ids, tr, cn
    # combine at the source rank: weighted top-8 sum over 7168-wide rows (the shape of the 64-rank configuration), 32 Ki tokens
    T, topk, d = 32768, 8, 7168
    yy = torch.empty((T * topk, d), dtype=torch.bfloat16, device=dev).normal_(generator=g)
    row_of = torch.randperm(T * topk, device=dev, generator=g).to(torch.int32).view(T, topk)
    gate = torch.rand((T, topk), device=dev, generator=g)
    oo = torch.empty((T, d), dtype=torch.bfloat16, device=dev)
    moe.moe_combine_topk_sum(yy, row_of, gate, out=oo)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        moe.moe_combine_topk_sum(yy, row_of, gate, out=oo)
    torch.cuda.synchronize()
    dtc = (time.perf_counter() - t0) / reps
    cbytes = (topk + 1) * 2 * d * T + 8 * T * topk
    out["combine_topk_sum"] = {"tokens": T, "topk": topk, "d": d, "bytes": cbytes, "us": dtc * 1e6, "GB_per_s": cbytes / dtc / 1e9,
                               "frac_hbm_peak": cbytes / dtc / 1e9 / HBM_PEAK_GBS, "bound": "hbm"}
    out["histogram_64_layers"] = {"bytes": nbytes, "GB_per_s": nbytes / dt / 1e9, "frac_hbm_peak": nbytes / dt / 1e9 / HBM_PEAK_GBS, "bound": "hbm"}
    return out


def ffn_granularity(moe, torch, np, wl):
    """(i) the same schedule issued as one call per slice (what per-matching launches would cost) beside the single
    call; (ii) expert time against the number of rows of a single slice -- this GPU's version of the paper's Figure 1."""
    out = {}
    cfg, x, y, offsets, S, E_loc, ffn_ws, w = wl.cfg, wl.x, wl.y, wl.offsets, wl.S, wl.cfg.E_loc, wl.ffn_ws, wl.w
    dev = x.device
    off_h = offsets.cpu().numpy().astype(np.int64)
    reps = 20 if cfg.d * cfg.f < (1 << 24) else 5

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps * 1e6

    one_call = timed(lambda: moe.moe_expert_ffn_sliced(x, offsets, S, E_loc, y=y, workspace=ffn_ws, **w))
    per_slice = []
    for sl in range(S):
        lo, hi = int(off_h[sl * E_loc]), int(off_h[(sl + 1) * E_loc])
        if hi > lo:
            o = torch.from_numpy((off_h[sl * E_loc:(sl + 1) * E_loc + 1] - lo).astype(np.int32)).to(dev)
            per_slice.append((x[lo:hi], o, y[lo:hi]))

    def run_slices():
        for xs, o, ys in per_slice:
            moe.moe_expert_ffn_sliced(xs, o, 1, E_loc, y=ys, workspace=ffn_ws, **w)

    out["ffn_one_call_us"] = one_call
    # the same call with the dispatch gather / combine scatter fused in: rows in a random arrival order, router weights
    g = torch.Generator(device=dev)
    g.manual_seed(3)
    M_used = int(off_h[-1])
    row_map = torch.randperm(M_used, device=dev, generator=g).to(torch.int32)
    gate = torch.rand((M_used,), device=dev, generator=g)
    out["ffn_one_call_row_map_us"] = timed(lambda: moe.moe_expert_ffn_sliced_mapped(x, offsets, S, E_loc, w["w_gate"], w["w_up"], w["w_down"],
                                                                                    row_map, gate, y=y, workspace=ffn_ws))
    out["ffn_one_call_per_slice_us"] = timed(run_slices)
    out["ffn_slices"] = len(per_slice)
    curve = {}
    for rows in (1, 8, 32, 64, 128, 256, 512, 1024, 2048, 4096, 8192):
        if rows > x.shape[0]:
            break
        o = torch.tensor([0, rows] + [rows] * (E_loc - 1), dtype=torch.int32, device=dev)      # all rows on local expert 0
        curve[str(rows)] = timed(lambda: moe.moe_expert_ffn_sliced(x[:rows], o, 1, E_loc, y=y[:rows], workspace=ffn_ws, **w))
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


class RowsView:
    """Stands in for x[M][d] when only some rows were copied back to the host: indexing with a subset of `rows`."""
    def __init__(self, data, rows, M):
        self.data, self.rows, self.shape = data, rows, (M, data.shape[1])

    def __getitem__(self, idx):
        import numpy as np
        pos = np.searchsorted(self.rows, idx)
        return self.data[pos]


def cpu_baseline(cfg, ids_h, r, x_sample, sample_rows, offsets_gpu, W, M):
    """The CPU oracle, as it stands, on the same workload: integer stages in full, the FFN on a bounded sample of rows
    (spread evenly over the schedule).  Reported in the metric's unit."""
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
    assert np.array_equal(offsets, offsets_gpu)
    sample = len(sample_rows)
    t0 = time.perf_counter()
    oracle.expert_ffn_sliced(RowsView(x_sample, sample_rows, M), offsets, cfg.E_loc, W, rows=sample_rows)
    t_ffn = time.perf_counter() - t0
    tflops = 6.0 * cfg.d * cfg.f * sample / t_ffn / 1e12
    return {"value": tflops, "unit": "TFLOP/s", "cores": int(blas_threads), "kind": "oracle",
            "sample": "FFN: %d of %d rows (evenly spaced) in float64 numpy (%.2f s, BLAS threads = cores); histogram %.1f ms, greedy %.2f ms, "
                      "BvN %.1f ms, slice table %.1f ms on the full workload, one thread each"
                      % (sample, M, t_ffn, t_hist * 1e3, t_greedy * 1e3, t_bvn * 1e3, t_slice * 1e3),
            "decompositions_per_s": {"greedy": 1.0 / t_greedy, "bvn": 1.0 / t_bvn}}


if __name__ == "__main__":
    main()

"""Seeded synthetic inputs for the MoE circuit-schedule path.

This module only draws random inputs and packs them into the byte layouts both
the CPU oracle and the GPU library consume.  It contains none of the method's
arithmetic (no histogramming, no matching, no FFN) and imports neither side.

The paper evaluates on routing traces of Mixtral / DeepSeek-MoE models running
MMLU and SPEED-Bench prompts (Section 4, "Datasets").  Those traces are not
available; the inputs below stand in for them: Zipf-distributed expert
popularity reproduces the sparse, skewed, imbalanced traffic of Section 2.2, a
small token count per rank plays the small-prompt regime and >= 8k tokens per
rank the large-prompt regime.

All bf16 / fp8 tensors are returned as raw bit patterns (numpy uint16 / uint8)
so that both consumers decode exactly the same bytes.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SEED_BASE = 26845 * 10


@dataclass(frozen=True)
class Config:
    """One named workload: routing shape, decomposition cap and expert FFN shape."""

    name: str
    index: int            # seed = SEED_BASE + index
    N: int                # ranks
    E: int                # experts in total (E % N == 0)
    topk: int             # experts per token
    T: int                # tokens per rank
    zipf_s: float
    kmax: int             # cap on greedy matchings
    d: int                # model width
    f: int                # FFN width
    weight_dtype: str     # "bf16" or "fp8"

    @property
    def E_loc(self) -> int:
        return self.E // self.N

    @property
    def seed(self) -> int:
        return SEED_BASE + self.index


CONFIGS = {
    "tiny": Config("tiny", 0, N=8, E=8, topk=2, T=512, zipf_s=1.2, kmax=4, d=256, f=512, weight_dtype="bf16"),
    "c2": Config("c2", 1, N=16, E=64, topk=2, T=4096, zipf_s=1.2, kmax=8, d=2048, f=1408, weight_dtype="bf16"),
    "c3": Config("c3", 2, N=8, E=8, topk=2, T=16384, zipf_s=0.8, kmax=4, d=4096, f=14336, weight_dtype="bf16"),
    "c4": Config("c4", 3, N=64, E=256, topk=8, T=8192, zipf_s=1.5, kmax=16, d=7168, f=2048, weight_dtype="fp8"),
}


# ----------------------------------------------------------------------------
# routing
# ----------------------------------------------------------------------------
def zipf_popularity(E: int, s: float, rng: np.random.Generator) -> np.ndarray:
    """p_e proportional to (rank(e)+1)^-s with a seeded random assignment of ranks to experts."""
    order = rng.permutation(E)
    p = (order.astype(np.float64) + 1.0) ** (-float(s))
    return p / p.sum()


def route_topk(N: int, T: int, E: int, topk: int, s: float, seed: int,
               per_rank_jitter: float = 0.0) -> np.ndarray:
    """Router output ids[N][T][topk] (int32): per token the top-k of log p + Gumbel noise,
    i.e. k experts sampled without replacement with probability proportional to p.
    per_rank_jitter > 0 multiplies p by lognormal(0, jitter) independently per source rank."""
    rng = np.random.default_rng(seed)
    p = zipf_popularity(E, s, rng)
    ids = np.empty((N, T, topk), dtype=np.int32)
    chunk = max(1, (1 << 22) // E)
    for n in range(N):
        pn = p
        if per_rank_jitter > 0.0:
            pn = p * rng.lognormal(0.0, per_rank_jitter, size=E)
            pn = pn / pn.sum()
        logp = np.log(pn)
        for t0 in range(0, T, chunk):
            t1 = min(T, t0 + chunk)
            g = rng.gumbel(size=(t1 - t0, E)) + logp
            if topk == 1:
                sel = np.argmax(g, axis=1)[:, None]
            else:
                part = np.argpartition(-g, topk - 1, axis=1)[:, :topk]
                key = np.take_along_axis(g, part, axis=1)
                sel = np.take_along_axis(part, np.argsort(-key, axis=1), axis=1)
            ids[n, t0:t1] = sel.astype(np.int32)
    return ids


def config_routing(cfg: Config, per_rank_jitter: float = 0.0) -> np.ndarray:
    return route_topk(cfg.N, cfg.T, cfg.E, cfg.topk, cfg.zipf_s, cfg.seed, per_rank_jitter)


def stress_matrices(B: int, N: int = 128, tokens_per_rank: int = 8192, topk: int = 8,
                    E: int = 512, seed: int = SEED_BASE + 4, zero_diag: bool = True) -> np.ndarray:
    """Batched decomposition stress input: B independent N x N int32 matrices.  Row i of a
    matrix ~ Multinomial(tokens_per_rank*topk, q) where q sums a Zipf(s) expert popularity
    over each rank's E/N experts and s ~ U[0.5, 2.0] per matrix.  Stands in for drawing
    every token's top-k route (6.9e10 draws at B=8192)."""
    rng = np.random.default_rng(seed)
    out = np.empty((B, N, N), dtype=np.int32)
    e_loc = E // N
    for b in range(B):
        s = rng.uniform(0.5, 2.0)
        p = zipf_popularity(E, s, rng)
        q = p.reshape(N, e_loc).sum(axis=1)
        m = rng.multinomial(tokens_per_rank * topk, q, size=N).astype(np.int32)
        if zero_diag:
            np.fill_diagonal(m, 0)
        out[b] = m
    return out


def random_matrices(B: int, N: int, seed: int, density: float = 1.0, high: int = 1000,
                    zero_diag: bool = False) -> np.ndarray:
    """Uniform random non-negative int32 test matrices with a given fill density; small value
    ranges (high) produce many equal-weight optima, which exercises tie-breaking."""
    rng = np.random.default_rng(seed)
    m = rng.integers(0, high, size=(B, N, N), dtype=np.int64)
    if density < 1.0:
        m = m * (rng.random((B, N, N)) < density)
    m = m.astype(np.int32)
    if zero_diag:
        for b in range(B):
            np.fill_diagonal(m[b], 0)
    return m


# ----------------------------------------------------------------------------
# bf16 / fp8 packing (format conversions of inputs only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16 bit patterns (uint16)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def _e4m3_table() -> np.ndarray:
    """All 256 OCP FP8 E4M3 values (bias 7, no infinities, S.1111.111 = NaN)."""
    t = np.empty(256, dtype=np.float64)
    for code in range(256):
        sign = -1.0 if code & 0x80 else 1.0
        e = (code >> 3) & 0xF
        m = code & 0x7
        if e == 0xF and m == 0x7:
            t[code] = np.nan
        elif e == 0:
            t[code] = sign * (m / 8.0) * 2.0 ** (-6)
        else:
            t[code] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return t


def f32_to_e4m3_bits(a: np.ndarray) -> np.ndarray:
    """Saturating round-to-nearest-even float32 -> OCP E4M3 codes (uint8), by nearest-value
    search over the 127 non-negative finite codes (ties to the even code)."""
    table = _e4m3_table()
    pos = table[:127]                       # codes 0..126: 0 .. 448, increasing
    x = np.asarray(a, dtype=np.float64)
    mag = np.minimum(np.abs(x), 448.0)
    hi = np.searchsorted(pos, mag, side="left").clip(0, 126)
    lo = (hi - 1).clip(0, 126)
    dlo = np.abs(mag - pos[lo])
    dhi = np.abs(pos[hi] - mag)
    pick_hi = (dhi < dlo) | ((dhi == dlo) & (hi % 2 == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    code = np.where(np.signbit(x), code | 0x80, code).astype(np.uint8)
    return code


@dataclass
class FFNWeights:
    """Expert weights in out-feature-major layout (the layout nn.Linear stores):
    w_gate, w_up: [E_loc][f][d]; w_down: [E_loc][d][f].
    bf16: uint16 bit patterns, scales None.
    fp8 : uint8 E4M3 codes plus float32 scales per 128x128 block,
          s_gate, s_up: [E_loc][f/128][d/128]; s_down: [E_loc][d/128][f/128];
          real weight = decode(code) * scale[block]."""

    dtype: str
    w_gate: np.ndarray
    w_up: np.ndarray
    w_down: np.ndarray
    s_gate: np.ndarray | None = None
    s_up: np.ndarray | None = None
    s_down: np.ndarray | None = None


def _quant_block128(w: np.ndarray):
    E, R, C = w.shape
    assert R % 128 == 0 and C % 128 == 0
    blk = w.reshape(E, R // 128, 128, C // 128, 128)
    amax = np.abs(blk).max(axis=(2, 4))
    scale = (amax / 448.0).astype(np.float32)
    scale = np.where(scale == 0, np.float32(1.0), scale).astype(np.float32)
    q = f32_to_e4m3_bits(blk / scale[:, :, None, :, None].astype(np.float64))
    return q.reshape(E, R, C), scale


def ffn_weights(E_loc: int, d: int, f: int, seed: int, dtype: str = "bf16", std: float = 0.02) -> FFNWeights:
    rng = np.random.default_rng(seed + 7919)
    wg = rng.standard_normal((E_loc, f, d), dtype=np.float32) * np.float32(std)
    wu = rng.standard_normal((E_loc, f, d), dtype=np.float32) * np.float32(std)
    wd = rng.standard_normal((E_loc, d, f), dtype=np.float32) * np.float32(std)
    if dtype == "bf16":
        return FFNWeights("bf16", f32_to_bf16_bits(wg), f32_to_bf16_bits(wu), f32_to_bf16_bits(wd))
    if dtype == "fp8":
        qg, sg = _quant_block128(wg)
        qu, su = _quant_block128(wu)
        qd, sd = _quant_block128(wd)
        return FFNWeights("fp8", qg, qu, qd, sg, su, sd)
    raise ValueError(dtype)


def activations(M: int, d: int, seed: int) -> np.ndarray:
    """x[M][d] ~ N(0,1) as bf16 bit patterns."""
    rng = np.random.default_rng(seed + 104729)
    out = np.empty((M, d), dtype=np.uint16)
    step = max(1, (1 << 24) // d)
    for r0 in range(0, M, step):
        r1 = min(M, r0 + step)
        out[r0:r1] = f32_to_bf16_bits(rng.standard_normal((r1 - r0, d), dtype=np.float32))
    return out


def ffn_weights_on_device(E_loc: int, d: int, f: int, seed: int, dtype: str, device, std: float = 0.02):
    """Expert weights drawn and packed on `device` with torch (same distribution and formats as ffn_weights(), another
    random stream): dict of w_gate, w_up [E_loc][f][d], w_down [E_loc][d][f] as bf16 tensors, or as uint8 E4M3 codes
    plus float32 scales s_* per 128 x 128 block (scale = amax / 448).  For timing runs whose host copy is not needed."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed + 7919)
    out = {}
    for name, shape in (("gate", (E_loc, f, d)), ("up", (E_loc, f, d)), ("down", (E_loc, d, f))):
        w = torch.randn(shape, dtype=torch.float32, device=device, generator=g) * std
        if dtype == "bf16":
            out["w_" + name] = w.to(torch.bfloat16)
            continue
        E, R, C = shape
        blk = w.view(E, R // 128, 128, C // 128, 128)
        scale = blk.abs().amax(dim=(2, 4)) / 448.0
        scale = torch.where(scale == 0, torch.ones_like(scale), scale)
        q = (blk / scale[:, :, None, :, None]).clamp(-448.0, 448.0).to(torch.float8_e4m3fn)
        out["w_" + name] = q.view(torch.uint8).view(E, R, C).contiguous()
        out["s_" + name] = scale.contiguous()
    return out


def activations_on_device(M: int, d: int, seed: int, device):
    """x[M][d] ~ N(0,1) as a bf16 torch tensor drawn on `device` (for row counts whose host copy would take minutes to
    draw and gigabytes to hold); a checker reads back the rows it needs.  Seeded, but a different stream than
    activations()."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed + 104729)
    out = torch.empty((M, d), dtype=torch.bfloat16, device=device)
    step = max(1, (1 << 26) // d)
    for r0 in range(0, M, step):
        r1 = min(M, r0 + step)
        out[r0:r1] = torch.randn((r1 - r0, d), dtype=torch.float32, device=device, generator=g).to(torch.bfloat16)
    return out


def random_offsets(n_groups: int, M: int, seed: int, empty_frac: float = 0.15, power: float = 2.0) -> np.ndarray:
    """Ragged group boundaries: int32[n_groups+1], non-decreasing, offsets[0]=0, last=M,
    with a share of empty groups.  Group sizes ~ u^power, u uniform: a larger power gives a few large groups
    among many small ones."""
    rng = np.random.default_rng(seed + 15485863)
    w = rng.random(n_groups) ** power
    w = w * (rng.random(n_groups) >= empty_frac)
    if w.sum() == 0:
        w[0] = 1.0
    sizes = np.floor(w / w.sum() * M).astype(np.int64)
    nz = np.flatnonzero(w)
    sizes[nz[0]] += M - sizes.sum()
    off = np.zeros(n_groups + 1, dtype=np.int32)
    off[1:] = np.cumsum(sizes)
    return off

// moe_expert_ffn_sliced: SwiGLU expert FFN over all (slice, expert) row groups of a schedule
// (Section 2.1 "compute"; Section 2.2: per-batch fixed overheads are what fragmenting
// decompositions pay, so all slices are issued by launches whose number does not depend on the
// number of matchings).
//
// Two grouped GEMMs on the bf16 MFMA units, persistent kernels looping over output tiles (for bf16 weights and 256-row
// blocks both run in one launch, phase-2 tiles waiting for the rows of H they read):
//   phase 1:  H = silu(X Wg^T) * (X Wu^T)     tile = BM rows x (128 gate + 128 up) columns
//   phase 2:  Y = H Wd^T                      tile = BM rows x 256 columns
// A tile never spans two (slice, expert) groups.  Both operands are K-contiguous, are copied
// global -> LDS in K slabs (2 to 4 in flight, XOR-swizzled 16-byte chunks; fp8 weights pass through
// registers to be dequantised) and read back as 16-byte MFMA fragments.  The weights feed the MFMA
// "A" port so that each lane ends up with 4 consecutive output columns of one row and can store
// 8 bytes at a time.  bf16 schedules with large groups run the adaptive-shape kernels (ffn_fused_kernel /
// ffn_adaptive_kernel), the others (and fp8 weights) the fixed-shape ffn_gemm_kernel.
// moe_expert_ffn_backward_sliced (the backward pass: the exchange of Section 2.1 repeated for the gradients) runs the
// same adaptive-shape kernels on other operands.
#include "common.hpp"
#include <type_traits>
#include <algorithm>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

constexpr int BN = 256;                // tile columns (phase 1: 128 gate + 128 up)
constexpr int PLAN_THREADS = 1024;
constexpr int MAX_GROUPS = 65536;
constexpr int PLAN_HDR = 5;            // plan[0] = (row blocks, 0, 0, 0); plan[1..2] / plan[3..4] = tile queue counters of phase 1 / 2

struct FfnArgs {
    const __bf16* x;                   // [M][d]
    __bf16* h;                         // [M][f]   workspace
    __bf16* y;                         // [M][d]
    const void *wg, *wu, *wd;          // bf16 or fp8 codes
    const float *sg, *su, *sd;         // block scales (fp8) or null
    int4* plan;                        // plan[0].x = number of row blocks; plan[PLAN_HDR + i] = (row0, row_end, expert, class)
    int d, f;
    const int32_t* row_map;            // [M] or null: row m of the schedule is row row_map[m] of x and of y
    const float* row_gate;             // [M] or null: y row is scaled by row_gate[m]
    int panel1, panel2;                // column groups per panel of the tile walk, phase 1 / phase 2 (see TileGeom)
    int* ready;                        // [row blocks] column units of h complete per row block (fused launch), zeroed by the plan kernel
    // The plain grouped GEMM of the adaptive-shape kernels' "phase 2": out[m][n] = sum_k A[m][k] * B_e[n][k] for the
    // rows m of every row block (expert e), n over NU units of 256 columns.  The forward pass sets A = h, B = w_down,
    // out = y; the backward pass runs it on other operands (see moe_expert_ffn_backward_sliced).
    struct Gemm {
        const __bf16* A; int lda;          // [rows][lda], K contiguous
        const __bf16* B; int ldb;          // B_e = B + e * strideB: [NU * 256][ldb], K contiguous
        long long strideB;
        __bf16* O; int ldo;
        int K, NU;
        const int4* etab;                  // or null.  Per expert (k0, K, r0, 0): the tile contracts over columns k0 .. k0 + K - 1 of
                                           // A and B, and row m of the schedule is row m - r0 of A
        int* queues;                       // 8 tile queue counters, zero at launch
    } g2;
    // backward pass, phase 1 with the gradient read-out (EPI == 1): dh in, [dg | du] and h out
    const __bf16* dh; int lddh;            // [M][lddh]
    __bf16* dgu;                           // [M][2 f]: dg in columns 0 .. f-1, du in f .. 2f-1
    int* queues1;                          // 8 tile queue counters of phase 1, zero at launch
};
// row of x that schedule row m reads (phase 1) / row of y it writes (phase 2)
__device__ __forceinline__ int mapped_row(const FfnArgs& a, int m) { return a.row_map ? a.row_map[m] : m; }

// ---------------------------------------------------------------------------------- plan kernel
// Splits every group into row blocks of BM rows.  One workgroup.  Malformed offsets cannot make
// it write outside the table: boundaries are clamped to [0, M] and to non-decreasing order, and
// entries beyond `cap` are dropped.
// Plan entry = (first row, end of the group, local expert, shape class of the block: 0 for more than 128 rows, else 1).
// The partial last blocks of the groups come first in the table and the full blocks after them: a partial block's
// tiles take longer than a full block's (they read twice the weights per MFMA), and a long tile handed out late is
// what the whole launch then waits for.  (A third class of 64 rows x 1024 columns for blocks of <= 64 rows was
// measured: its tiles take twice as long as any other and made phase 1 of the bench schedule 7 % slower by finishing
// last; it is not in the kernel.)
__device__ __forceinline__ int plan_scan(int v, int tid, int* wave_tot, int& total) {       // exclusive prefix over the workgroup
    const int lane = tid & 63, wave = tid >> 6;
    int incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int o = __shfl_up(incl, off);
        if (lane >= off) incl += o;
    }
    __syncthreads();
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int base = 0;
    total = 0;
    for (int w = 0; w < PLAN_THREADS / 64; ++w) {
        if (w < wave) base += wave_tot[w];
        total += wave_tot[w];
    }
    return base + incl - v;
}

// two prefixes behind one pair of barriers
__device__ __forceinline__ void plan_scan2(int a, int b, int tid, int* wave_a, int* wave_b, int& excl_a, int& excl_b, int& total_a,
                                           int& total_b) {
    const int lane = tid & 63, wave = tid >> 6;
    int ia = a, ib = b;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int oa = __shfl_up(ia, off), ob = __shfl_up(ib, off);
        if (lane >= off) { ia += oa; ib += ob; }
    }
    __syncthreads();
    if (lane == 63) { wave_a[wave] = ia; wave_b[wave] = ib; }
    __syncthreads();
    int base_a = 0, base_b = 0;
    total_a = 0; total_b = 0;
    for (int w = 0; w < PLAN_THREADS / 64; ++w) {
        if (w < wave) { base_a += wave_a[w]; base_b += wave_b[w]; }
        total_a += wave_a[w]; total_b += wave_b[w];
    }
    excl_a = base_a + ia - a;
    excl_b = base_b + ib - b;
}
__global__ __launch_bounds__(PLAN_THREADS)
void ffn_plan_kernel(const int32_t* __restrict__ offsets, int G, int e_loc, int M, int bm, int cap, int4* __restrict__ plan,
                     int* __restrict__ ready) {
    __shared__ int wave_tot[PLAN_THREADS / 64], wave_tot2[PLAN_THREADS / 64];
    const int tid = threadIdx.x;
    auto bounds = [&](int g, int& lo, int& hi) {
        lo = hi = 0;
        if (g < G) {
            lo = min(max(offsets[g], 0), M);
            hi = min(max(offsets[g + 1], lo), M);
        }
    };
    // ---- number of partial blocks (groups whose size is not a multiple of bm); with at most one group per thread
    //      the scan of the table pass below yields it
    int n_partial = 0;
    if (G > PLAN_THREADS) {
        int partial = 0;
        for (int g = tid; g < G; g += PLAN_THREADS) {
            int lo, hi;
            bounds(g, lo, hi);
            partial += (hi - lo) % bm != 0;
        }
        plan_scan(partial, tid, wave_tot, n_partial);
    }
    // ---- table: partial blocks in group order, then the full blocks in group order
    int run_partial = 0, run_full = n_partial;                        // (uniform: every thread adds the same totals)
    for (int g0 = 0; g0 < G; g0 += PLAN_THREADS) {
        const int g = g0 + tid;
        int lo, hi;
        bounds(g, lo, hi);
        const int rows = hi - lo, nfull = rows / bm, has_partial = rows % bm != 0;
        int ex_partial, ex_full, tot_partial, tot_full;
        plan_scan2(has_partial, nfull, tid, wave_tot, wave_tot2, ex_partial, ex_full, tot_partial, tot_full);
        if (G <= PLAN_THREADS) run_full = tot_partial;               // the only pass: all partial blocks are known now
        const int at_partial = run_partial + ex_partial;
        run_partial += tot_partial;
        int at_full = run_full + ex_full;
        run_full += tot_full;
        for (int k = 0; k < nfull; ++k, ++at_full)
            if (at_full < cap) plan[PLAN_HDR + at_full] = make_int4(lo + k * bm, hi, g % e_loc, bm > 128 ? 0 : 1);
        if (has_partial && at_partial < cap) {
            const int row = lo + nfull * bm;
            plan[PLAN_HDR + at_partial] = make_int4(row, hi, g % e_loc, hi - row > 128 ? 0 : 1);
        }
    }
    for (int i = tid; i < min(run_full, cap); i += PLAN_THREADS) ready[i] = 0;      // per row block: column units of h complete
    if (tid == 0) plan[0] = make_int4(min(run_full, cap), 0, 0, 0);
    if (tid >= 1 && tid < PLAN_HDR) plan[tid] = make_int4(0, 0, 0, 0);      // tile queue counters
}

// ---------------------------------------------------------------------------------- helpers
// g * sigmoid(g) with the hardware reciprocal (1 ulp) instead of an IEEE division: the result is rounded to bf16 anyway,
// and the division's dozen instructions per value were a visible part of a tile's read-out
__device__ __forceinline__ float silu(float g) { return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)); }

__device__ __forceinline__ u32x2 pack4(float a, float b, float c, float d) {
    bf16x4 v = {(__bf16)a, (__bf16)b, (__bf16)c, (__bf16)d};
    return __builtin_bit_cast(u32x2, v);
}

// 8 consecutive OCP FP8 E4M3 codes (8 bytes; bias 7, subnormals at exponent field 0, no infinities, S.1111.111 = NaN)
// times one scale -> 8 bf16.  gfx950 decodes two codes per v_cvt_pk_f32_fp8.
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32x4 dequant8(u32x2 codes, float scale) {
    const f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)codes.x, false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)codes.x, true);
    const f32x2 c = __builtin_amdgcn_cvt_pk_f32_fp8((int)codes.y, false), d = __builtin_amdgcn_cvt_pk_f32_fp8((int)codes.y, true);
    bf16x8 o = {(__bf16)(a.x * scale), (__bf16)(a.y * scale), (__bf16)(b.x * scale), (__bf16)(b.y * scale),
                (__bf16)(c.x * scale), (__bf16)(c.y * scale), (__bf16)(d.x * scale), (__bf16)(d.y * scale)};
    return __builtin_bit_cast(u32x4, o);
}

// ---------------------------------------------------------------------------------- GEMM kernel
// PHASE 1: A = x (K = d), B rows 0..127 = gate rows, 128..255 = up rows of the tile's 128 columns.
// PHASE 2: A = h (K = f), B rows = 256 rows of w_down.
// MB = row blocks of 32 per wavefront: BM = 64 * MB.   FP8 = weights are block-scaled E4M3 codes.
//
// K slabs of 64 are double buffered in LDS.  bf16 operands go global -> LDS directly (each
// wavefront instruction deposits 64 x 16 bytes contiguously, so the XOR swizzle is applied to
// the global chunk a lane fetches); fp8 weights pass through registers to be dequantised.
// Tiles are handed out by eight atomic queues, one per XCD (workgroup id modulo 8), each
// walking its own chunks of neighbouring tiles so that the workgroups sharing an L2 also share
// operand slabs; a workgroup whose queue runs dry takes from the others.

struct TileGeom {                      // how tiles are grouped into chunks, and the order in which the chunks are walked
    int nblocks, NT, NCG, CN, RB, NRG, W, nchunks;
    __device__ __forceinline__ void init(int nblocks_, int NT_, int panel) {
        nblocks = nblocks_; NT = NT_;
        NCG = (NT + 7) / 8;                        // column groups of at most 8 (11 -> 2 x 6)
        CN = (NT + NCG - 1) / NCG;
        RB = 32 / CN < 1 ? 1 : 32 / CN;            // about 32 tiles per chunk
        NRG = (nblocks + RB - 1) / RB;             // row groups
        W = panel < 1 ? 1 : (panel > NCG ? NCG : panel);      // column groups per panel
        nchunks = NRG * NCG;
    }
    // ticket k of queue x -> tile; returns 1 = valid, 0 = hole in the padded grid, -1 = queue exhausted.
    // Chunks are walked panel by panel: inside a panel of W column groups the row groups are the outer loop, so the
    // panel's weights are touched again after one row group's worth of other traffic and stay in the memory-side cache
    // while the activations stream past; W = NCG (one panel) when an expert's weights are small.
    __device__ __forceinline__ int decode(int x, int k, int& blk, int& nt) const {
        const int chs = RB * CN;
        const int c = (k / chs) * 8 + x, j = k % chs;
        if (c >= nchunks) return -1;
        const int full = (NCG / W) * W;            // column groups inside whole panels
        const int c0 = NRG * full;
        int rg, cg;
        if (c < c0) {
            const int per = NRG * W, p = c / per, rem = c - p * per;
            rg = rem / W; cg = p * W + rem - rg * W;
        } else {
            const int wl = NCG - full, rem = c - c0;
            rg = rem / wl; cg = full + rem - rg * wl;
        }
        blk = rg * RB + j / CN;
        nt = cg * CN + j % CN;
        return (blk < nblocks && nt < NT) ? 1 : 0;
    }
};

template <int N> __device__ __forceinline__ void wait_vmcnt();
#define MOE_WAIT_VMCNT(n) template <> __device__ __forceinline__ void wait_vmcnt<n>() { asm volatile("s_waitcnt vmcnt(" #n ")" ::: "memory"); }
MOE_WAIT_VMCNT(0) MOE_WAIT_VMCNT(1) MOE_WAIT_VMCNT(2) MOE_WAIT_VMCNT(3) MOE_WAIT_VMCNT(4) MOE_WAIT_VMCNT(5) MOE_WAIT_VMCNT(6) MOE_WAIT_VMCNT(7) 
MOE_WAIT_VMCNT(8) MOE_WAIT_VMCNT(9) MOE_WAIT_VMCNT(10) MOE_WAIT_VMCNT(11) MOE_WAIT_VMCNT(12) MOE_WAIT_VMCNT(13) MOE_WAIT_VMCNT(14) MOE_WAIT_VMCNT(15) 
MOE_WAIT_VMCNT(16) MOE_WAIT_VMCNT(17) MOE_WAIT_VMCNT(18) MOE_WAIT_VMCNT(19) MOE_WAIT_VMCNT(20) MOE_WAIT_VMCNT(21) MOE_WAIT_VMCNT(22) MOE_WAIT_VMCNT(23) 
MOE_WAIT_VMCNT(24) MOE_WAIT_VMCNT(25) MOE_WAIT_VMCNT(26) MOE_WAIT_VMCNT(27) MOE_WAIT_VMCNT(28) MOE_WAIT_VMCNT(29) MOE_WAIT_VMCNT(30) MOE_WAIT_VMCNT(31) 
MOE_WAIT_VMCNT(32) MOE_WAIT_VMCNT(33) MOE_WAIT_VMCNT(34) MOE_WAIT_VMCNT(35) MOE_WAIT_VMCNT(36) MOE_WAIT_VMCNT(37) MOE_WAIT_VMCNT(38) MOE_WAIT_VMCNT(39) 
MOE_WAIT_VMCNT(40) MOE_WAIT_VMCNT(41) MOE_WAIT_VMCNT(42) MOE_WAIT_VMCNT(43) MOE_WAIT_VMCNT(44) MOE_WAIT_VMCNT(45) MOE_WAIT_VMCNT(46) MOE_WAIT_VMCNT(47) 
MOE_WAIT_VMCNT(48) MOE_WAIT_VMCNT(49) MOE_WAIT_VMCNT(50) MOE_WAIT_VMCNT(51) MOE_WAIT_VMCNT(52) MOE_WAIT_VMCNT(53) MOE_WAIT_VMCNT(54) MOE_WAIT_VMCNT(55) 
MOE_WAIT_VMCNT(56) MOE_WAIT_VMCNT(57) MOE_WAIT_VMCNT(58) MOE_WAIT_VMCNT(59) MOE_WAIT_VMCNT(60) MOE_WAIT_VMCNT(61) MOE_WAIT_VMCNT(62) MOE_WAIT_VMCNT(63) 
#undef MOE_WAIT_VMCNT

// Workgroup barrier that orders LDS traffic only.  (__syncthreads() also drains every outstanding global
// access, which would serialise the slab copies that are meant to stay in flight across K steps.)
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// BK = K slab width (32 or 64 bf16), NST = LDS stages: slabs kt+1 .. kt+NST-1 are in flight or landed while slab kt
// is multiplied.
// WMW = wavefronts along the rows (2 or 4; always 2 along the columns), MB = 32-row blocks per wavefront:
// BM = 32 * MB * WMW rows per tile, 128 * WMW threads.  Eight wavefronts (two per SIMD) matter because one
// wavefront can only issue slab copies at a limited rate: with four, the copies, not the MFMAs, set the pace.
template <int PHASE, int WMW, int MB, bool FP8, int BK, int NST, int PER_CU>
__global__ __launch_bounds__(WMW * 128, PER_CU)
void ffn_gemm_kernel(FfnArgs a) {
    constexpr int FFN_THREADS = WMW * 128;
    constexpr int BM = 32 * MB * WMW;
    constexpr int ROW_BYTES = BK * 2;                  // one slab row
    constexpr int CPR = BK / 8;                        // 16-byte chunks per row (4 or 8)
    constexpr int RS = FFN_THREADS / CPR;              // slab rows covered by one pass of all threads
    constexpr int KS = BK / 16;                        // MFMA K steps per slab
    constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES, STAGE = A_BYTES + B_BYTES;
    constexpr int CA = BM / RS;                        // 16-byte chunks per thread, A slab
    constexpr int CB = BN / RS;                        // B slab
    constexpr int ESZ = FP8 ? 1 : 2;
    constexpr int LPS = CA + (FP8 ? 0 : CB);           // asynchronous copies per thread and slab
    static_assert(NST >= 2 && NST <= 4 && KS % 2 == 0 && 3 * LPS < 64, "pipeline shape");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ int s_ticket[2];                        // (block, column tile) of the next tile, -1 = none

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l31 = lane & 31, lhi = lane >> 5;
    const int K = PHASE == 1 ? a.d : a.f;
    const int KT = K / BK;
    TileGeom geom;
    geom.init(a.plan[0].x, PHASE == 1 ? a.f / 128 : a.d / BN, PHASE == 1 ? a.panel1 : a.panel2);
    int* queues = (int*)(a.plan + (PHASE == 1 ? 1 : 3));
    const int my_xcd = blockIdx.x & 7;

    // LDS layout of a slab: row-major, 16-byte chunk c of row r sits at position c ^ swz(r).  With 64 banks of 4
    // bytes a 16-lane group of a ds_read_b128 touches 256 bytes; swz makes 16 consecutive rows hit 16 different
    // 16-byte bank groups: 128-byte rows -> (r >> 1) & 7, 64-byte rows -> (r >> 2) & 3.
    // Staging: chunk id = tid + i*threads -> row = tid / CPR + i*RS.  One wavefront instruction deposits 64 x 16 bytes
    // contiguously (whole rows), so the swizzle is applied to the global chunk a lane fetches.
    const int row0 = tid / CPR;
    const int swz0 = BK == 64 ? ((row0 >> 1) & 7) : ((row0 >> 2) & 3);     // same for row0 + i*RS
    const int kcg = (tid % CPR) ^ swz0;
    const int wave_bytes = wave * 1024;
    const int st_off = row0 * ROW_BYTES + ((tid % CPR) << 4);    // register path: same position
    // fragment coordinates: row l31 of a 32-row block, chunk (2*ks + lhi)
    const int fswz = BK == 64 ? ((l31 >> 1) & 7) : ((l31 >> 2) & 3);
    int frag_off[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) frag_off[ks] = l31 * ROW_BYTES + ((((ks << 1) | lhi) ^ fswz) << 4);
    int brow[4];                                       // first B-slab row of this wave's 4 column blocks
#pragma unroll
    for (int q = 0; q < 4; ++q) brow[q] = PHASE == 1 ? ((q >> 1) * 128 + wn * 64 + (q & 1) * 32) : (wn * 128 + q * 32);

    // thread 0 pulls tickets; own queue first, then the others
    auto fetch = [&](int first_k) {
        int q = my_xcd, k = first_k, blk = -1, nt = -1;
        for (int tries = 0; tries < 8;) {
            int st = geom.decode(q, k, blk, nt);
            if (st == 1) break;
            if (st < 0) { blk = -1; ++tries; q = (q + 1) & 7; }
            if (tries < 8) k = atomicAdd(&queues[q], 1);
        }
        s_ticket[0] = blk; s_ticket[1] = nt;
    };
    if (tid == 0) fetch(atomicAdd(&queues[my_xcd], 1));
    __syncthreads();
    if (s_ticket[0] < 0) return;

    // ---- per-tile state (set by setup()): global addressing of the slab copies; rows past the group's end re-read
    //      its last row.  B slab row r = row0 + RS*i: only i selects gate / up / 128-row block, so each B address is
    //      a wave-uniform base plus one per-thread byte offset.
    const __bf16* Abase = (PHASE == 1 ? a.x : (const __bf16*)a.h);
    const unsigned int b_voff = (unsigned int)(row0 * K + kcg * 8) * ESZ;
    int m0 = 0, m_end = 0, nt = 0;
    long long a_off[CA];                               // element offset of this thread's chunk (64 bit: M * K may pass 2^31)
    const unsigned char* bbase[CB];
    const float* sbase[CB];
    auto setup = [&](int blk, int nt_) {
        const int4 info = a.plan[PLAN_HDR + blk];
        m0 = info.x; m_end = info.y; nt = nt_;
        const int e = info.z;
        const int rows = min(BM, m_end - m0);
#pragma unroll
        for (int i = 0; i < CA; ++i) {
            const int m = m0 + min(row0 + RS * i, rows - 1);
            a_off[i] = (long long)(PHASE == 1 ? mapped_row(a, m) : m) * K + kcg * 8;
        }
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            constexpr int PER_HALF = 128 / RS;                            // passes per 128 slab rows
            long long wrow;                                               // first weight row of this strip
            const void* w;
            if (PHASE == 1) { wrow = (long long)e * a.f + nt * 128 + RS * (i % PER_HALF); w = (i < PER_HALF) ? a.wg : a.wu; }
            else            { wrow = (long long)e * a.d + nt * BN + RS * i;                 w = a.wd; }
            bbase[i] = (const unsigned char*)w + wrow * K * ESZ;
            if (FP8) {
                // scale row of the 128 x 128 block holding the strip
                if (PHASE == 1) sbase[i] = ((i < PER_HALF) ? a.sg : a.su) + ((long long)e * (a.f / 128) + nt) * (K / 128);
                else            sbase[i] = a.sd + ((long long)e * (a.d / 128) + nt * 2 + i / PER_HALF) * (K / 128);
            } else {
                sbase[i] = nullptr;
            }
        }
    };

    // asynchronous global -> LDS copies of one slab (A always; B when it is bf16)
    auto issue_slab = [&](int kt, int stage) {
        unsigned char* sa = smem + stage * STAGE + wave_bytes;
        unsigned char* sb = sa + A_BYTES;
#pragma unroll
        for (int i = 0; i < CA; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Abase + a_off[i] + kt * BK),
                                             (__attribute__((address_space(3))) void*)(sa + i * RS * ROW_BYTES), 16, 0, 0);
        if (!FP8) {
#pragma unroll
            for (int i = 0; i < CB; ++i)
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)(bbase[i] + (size_t)kt * BK * ESZ + b_voff),
                    (__attribute__((address_space(3))) void*)(sb + i * RS * ROW_BYTES), 16, 0, 0);
        }
    };
    // fp8 weights: codes through registers (one slab ahead), dequantised on the way into LDS
    u32x2 rb[CB];
    float rscale[CB];
    auto load_b_regs = [&](int kt) {
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            rb[i] = *reinterpret_cast<const u32x2*>(bbase[i] + (size_t)kt * BK + b_voff);
            rscale[i] = sbase[i][(kt * BK) >> 7];
        }
    };
    auto store_b_regs = [&](int stage) {
        unsigned char* sb = smem + stage * STAGE + A_BYTES;
#pragma unroll
        for (int i = 0; i < CB; ++i) *reinterpret_cast<u32x4*>(sb + st_off + i * RS * ROW_BYTES) = dequant8(rb[i], rscale[i]);
    };

    // ---- K loop, software pipelined.  All NST stages are kept busy: the barrier that lets a wavefront read
    //      slab kt+1 sits before the last MFMA batch of slab kt; by then every wavefront holds all of slab kt
    //      in registers, so the same barrier frees slab kt's stage for slab kt+NST.
    auto load_frags = [&](bf16x8 (&wf)[4], bf16x8 (&xf)[MB], int stage, int ks) {
        const unsigned char* sa = smem + stage * STAGE + (wm * (MB * 32)) * ROW_BYTES;
        const unsigned char* sb = smem + stage * STAGE + A_BYTES;
#pragma unroll
        for (int q = 0; q < 4; ++q) wf[q] = *reinterpret_cast<const bf16x8*>(sb + brow[q] * ROW_BYTES + frag_off[ks]);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) xf[mb] = *reinterpret_cast<const bf16x8*>(sa + mb * 32 * ROW_BYTES + frag_off[ks]);
    };
    auto load_frag_one = [&](bf16x8 (&wf)[4], bf16x8 (&xf)[MB], int stage, int ks, int i) {
        const unsigned char* sa = smem + stage * STAGE + (wm * (MB * 32)) * ROW_BYTES;
        const unsigned char* sb = smem + stage * STAGE + A_BYTES;
        if (i < 4) wf[i] = *reinterpret_cast<const bf16x8*>(sb + brow[i] * ROW_BYTES + frag_off[ks]);
        else       xf[i - 4] = *reinterpret_cast<const bf16x8*>(sa + (i - 4) * 32 * ROW_BYTES + frag_off[ks]);
    };
    auto issue_one = [&](int kt, int stage, int i) {
        unsigned char* sa = smem + stage * STAGE + wave_bytes;
        unsigned char* sb = sa + A_BYTES;
        if (i < CA)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Abase + a_off[i] + kt * BK),
                                             (__attribute__((address_space(3))) void*)(sa + i * RS * ROW_BYTES), 16, 0, 0);
        else
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(bbase[i - CA] + (size_t)kt * BK * ESZ + b_voff),
                (__attribute__((address_space(3))) void*)(sb + (i - CA) * RS * ROW_BYTES), 16, 0, 0);
    };
    // wait until at most `y` whole slabs of this thread's copies are outstanding (copies complete in order)
    auto wait_slabs = [&](int y) {
        if (y >= 3) wait_vmcnt<3 * LPS>(); else if (y == 2) wait_vmcnt<2 * LPS>();
        else if (y == 1) wait_vmcnt<LPS>(); else wait_vmcnt<0>();
    };

    // first slabs of a tile (all stages must be free)
    auto prologue = [&]() {
        if (FP8) { load_b_regs(0); store_b_regs(0); if (KT > 1) load_b_regs(1); }
#pragma unroll
        for (int j = 0; j < NST; ++j)
            if (j < KT) issue_slab(j, j);
    };

    setup(s_ticket[0], s_ticket[1]);
    prologue();
    while (true) {
        f32x16 acc[MB][4];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mb][q][v] = 0.f;

        wait_slabs(min(NST - 1, KT - 1));
        lds_barrier();                   // slab 0 of this tile is in LDS; everybody has read the ticket of this tile
        if (tid == 0) fetch(atomicAdd(&queues[my_xcd], 1));             // ticket of the next tile
        bf16x8 wf[2][4], xf[2][MB];
        load_frags(wf[0], xf[0], 0, 0);

        // One slab.  ISSUE = a further slab (kt + NST) exists and is fetched; the steady-state body is branch free so
        // that the scheduler can spread LDS reads and slab copies between the MFMAs (MFMA first: the wait for the
        // fragments of this batch must not also wait for reads issued for the next one).
        auto slab = [&](int kt, auto issue_tag) {
            constexpr bool ISSUE = decltype(issue_tag)::value;
            const int stage = kt % NST;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const int cur = ks & 1, nxt = cur ^ 1;
                bool copies = false;
                if (ks + 1 < KS) {
                    load_frags(wf[nxt], xf[nxt], stage, ks + 1);
                } else if (ISSUE) {
                    if (FP8) store_b_regs((kt + 1) % NST);
                    wait_vmcnt<(NST - 2) * LPS>();                       // slab kt+1 landed; kt+2 .. kt+NST-1 may be in flight
                    lds_barrier();
                    if (FP8) load_b_regs(kt + 2);                        // before the copies: waited for first
                    // fragment reads and slab copies alternate in program order (a copy writes LDS, so the compiler
                    // keeps it ordered against the reads around it)
                    constexpr int NF = 4 + MB, NC = CA + (FP8 ? 0 : CB);
#pragma unroll
                    for (int i = 0; i < (NF > NC ? NF : NC); ++i) {
                        if (i < NF) load_frag_one(wf[nxt], xf[nxt], (kt + 1) % NST, 0, i);
                        if (i < NC) issue_one(kt + NST, stage, i);
                    }
                    copies = true;
                } else if (kt + 1 < KT) {
                    if (FP8) store_b_regs((kt + 1) % NST);
                    wait_slabs(min(NST - 2, KT - 2 - kt));
                    lds_barrier();
                    load_frags(wf[nxt], xf[nxt], (kt + 1) % NST, 0);
                    if (FP8 && kt + 2 < KT) load_b_regs(kt + 2);
                }
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        acc[mb][q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[cur][q], xf[cur][mb], acc[mb][q], 0, 0, 0);
                // issue order: one MFMA, then at most one LDS read and one slab copy, repeated
                constexpr int NMF = 4 * MB, NFR = 4 + MB, NCP = CA + CB;
                if (copies) {
#pragma unroll
                    for (int i = 0; i < (NMF > NFR ? NMF : NFR); ++i) {
                        if (i < NMF) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
                        if (i < NFR) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // LDS read
                        if (i < NCP) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);   // vector memory (slab copy)
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < (NMF > NFR ? NMF : NFR); ++i) {
                        if (i < NMF) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        if (i < NFR) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        {
            int kt = 0;
            for (; kt + NST < KT; ++kt) slab(kt, std::true_type{});
            for (; kt < KT; ++kt) slab(kt, std::false_type{});
        }
        lds_barrier();                   // every fragment is in registers: all stages are free; next ticket visible
        const int em0 = m0, em_end = m_end, ent = nt;
        const int nblk = s_ticket[0], nnt = s_ticket[1];
        if (nblk >= 0) { setup(nblk, nnt); prologue(); }                // the next tile's first slabs fly during the epilogue


        // ---- epilogue.  acc[mb][q][v]: row m = l31 of row block mb; column n = 8*(v>>2) + 4*lhi + (v&3)
        //      of column block q
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int m = em0 + wm * (MB * 32) + mb * 32 + l31;
            if (m < em_end) {
                if (PHASE == 1) {
                    __bf16* out = a.h + (long long)m * a.f + ent * 128 + wn * 64 + 4 * lhi;
#pragma unroll
                    for (int q = 0; q < 2; ++q)
#pragma unroll
                        for (int vg = 0; vg < 4; ++vg) {
                            float hv[4];
#pragma unroll
                            for (int j = 0; j < 4; ++j) hv[j] = silu(acc[mb][q][vg * 4 + j]) * acc[mb][q + 2][vg * 4 + j];
                            *reinterpret_cast<u32x2*>(out + q * 32 + vg * 8) = pack4(hv[0], hv[1], hv[2], hv[3]);
                        }
                } else {
                    __bf16* out = a.y + (long long)mapped_row(a, m) * a.d + ent * BN + wn * 128 + 4 * lhi;
                    const float gate = a.row_gate ? a.row_gate[m] : 1.0f;
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int vg = 0; vg < 4; ++vg)
                            *reinterpret_cast<u32x2*>(out + q * 32 + vg * 8) =
                                pack4(gate * acc[mb][q][vg * 4], gate * acc[mb][q][vg * 4 + 1], gate * acc[mb][q][vg * 4 + 2],
                                      gate * acc[mb][q][vg * 4 + 3]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);     // one row block at a time: keeps the accumulator read-out short-lived
        }
        if (nblk < 0) break;
    }
}

// ---------------------------------------------------------------------------------- adaptive-shape GEMM kernel (bf16)
// Same dataflow as ffn_gemm_kernel with 8 wavefronts of 64 x 128 each, but the arrangement of the wavefronts is chosen
// per row block so that ragged slices do not pay for 256 rows they do not have:
//   class 0: 4 x 2 wavefronts = 256 rows x 256 columns;  64-wide K slabs (128-byte rows) of 64 KiB, two in LDS
//   class 1: 2 x 4            = 128 rows x 512 columns;  32-wide K slabs (64-byte rows) of 40 KiB, three in LDS
// Both classes run the same number of MFMAs per tile.  (A 1 x 8 arrangement of 64 rows x 1024 columns was measured
// too: its tiles read four times the weights per row and take twice as long as the others -- see the plan kernel.)
// Columns come in units (phase 1: 128 hidden units = 128 gate + 128 up rows; phase 2: 256 rows of w_down); a tile of
// class c covers 1 / 2 consecutive units.  A unit past the end is fetched as the last valid one and not stored.
// The 256-row class, which does most of the work, has 128-byte slab rows so that every copy fetches whole cache
// lines: a 64-byte row is half a line whose other half is requested again by the next slab, which doubles the
// requests to the L2 and the fill traffic into the L1 and keeps the address FIFO of the memory pipeline full (and
// the MFMAs queued behind a copy waiting) for a fifth of the time.
// The barrier at the end of slab s publishes slab s + 1 and frees the buffer of slab s; the copies of slab s + NSS
// go out from there on, spaced between the MFMAs (slot 0 = rest of slab s, slot i = K step i - 1 of slab s + 1).
constexpr int NW = 8;                                         // wavefronts per workgroup
template <int CLS> struct Cls {
    static_assert(CLS == 0 || CLS == 1, "two shape classes");
    static constexpr int WMW = (CLS == 0 ? 4 : 2) * NW / 8, WNW = NW / WMW;
    static constexpr int MB = 16 / NW, NQ = 4;                                    // 32-row / 32-column blocks per wavefront
    static constexpr int BMc = 32 * MB * WMW, BNc = 32 * NQ * WNW;
    static constexpr int U = BNc / 256;                                     // column units per tile
    static constexpr int ROWB = CLS == 0 ? 128 : 64;                        // bytes per slab row
    static constexpr int SUB = ROWB / 32;                                   // MFMA K steps (of 16) per slab
    static constexpr int RPC = NW * 1024 / ROWB;                                 // slab rows one copy of the workgroup deposits
    static constexpr int A_BYTES = BMc * ROWB, B_BYTES = BNc * ROWB, SLAB = A_BYTES + B_BYTES;
    static constexpr int NSS = CLS == 1 ? 3 : 2;                            // slabs resident in LDS
    static constexpr int CA = BMc / RPC, CB = BNc / RPC, NCOPY = CA + CB;   // copies per wavefront and slab
    // copies per slot (slot 0, 1, 2; none later)
    static constexpr int S0 = (CLS == 0 ? 4 : 3) * 8 / NW, S1 = NCOPY - S0, S2 = 0;
    static_assert(S0 + S1 + S2 == NCOPY && (S2 == 0 || SUB > 2) && (S1 == 0 || SUB > 1), "the slots hold every copy and end before the next slab's last K step");
};
constexpr int STAGE_OFF = 131072;                             // slab buffers below (2 x 64 KiB >= 3 x 40 KiB), output staging above
constexpr int STAGE_WAVE = 4096;                              // staging per wavefront: 32 rows x 128 bytes
constexpr int ADAPTIVE_LDS = STAGE_OFF + NW * STAGE_WAVE;      // 160 KiB: all of a compute unit's LDS

// GATHER (phase 1 with a row map): the rows of a tile lie anywhere in x, so every thread carries the 64-bit address of
// its rows; otherwise the rows of a tile are consecutive and one buffer descriptor per tile (64-bit base at the
// tile's first row) plus 32-bit offsets inside the tile address them, whatever the size of the operand.
// FUSED (both phases in one launch, see ffn_fused_kernel): a phase-1 tile, once its rows of h are stored, adds the
// column units it covered to the ready counter of its row block; a phase-2 ticket is handed to the workgroup only when
// the counter of its row block has reached the number of column units of h.  The hidden activations cross from one
// workgroup to another inside the launch, possibly from one die's L2 to another's: their stores (phase 1) and their
// loads (phase 2) are issued at device scope (the sc1 bit of the instruction: the store is written through to where
// every die sees it before it counts as complete, the load does not take a copy that is private to its die), and the
// counters are device-scope atomics; a writer signals after all its stores have completed (vmcnt(0) in every wavefront,
// then a barrier), a reader issues its loads after it has seen the count.
constexpr int DEVICE_SCOPE = 16;       // cache-policy bit sc1 of a buffer instruction
// EPI (phase 1): 0 = h = silu(g) * u is stored; 1 = the backward pass: with dh read from memory, dg = dh * u * silu'(g) and
// du = dh * silu(g) are stored side by side and h beside them.
template <int PHASE, bool GATHER, bool FUSED, int EPI = 0>
__device__ __forceinline__ void ffn_adaptive_body(const FfnArgs& a, unsigned char* smem) {
    static_assert(PHASE == 1 || !GATHER, "only phase 1 gathers its rows");
    static_assert(EPI == 0 || (PHASE == 1 && !FUSED), "the gradient read-out belongs to phase 1 of a launch of its own");
    // next tile: (block, tile index, class, first row, end row, expert); block -1 = none.  It shares its bytes with
    // wavefront 0's output staging: written by that wavefront after its read-out, read by the others before the
    // next read-out begins (inside the slab loop, or ahead of a barrier).
    int* const s_ticket = reinterpret_cast<int*>(smem + STAGE_OFF);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l31 = lane & 31, lhi = lane >> 5;
    int K = PHASE == 1 ? a.d : a.g2.K;                          // (per tile when the GEMM has an expert table)
    const int NU = PHASE == 1 ? a.f / 128 : a.g2.NU;            // column units
    const int lda = PHASE == 1 ? a.d : a.g2.lda, ldb = PHASE == 1 ? a.d : a.g2.ldb;      // row pitch of the operands, elements
    TileGeom geom;
    geom.init(a.plan[0].x, NU, PHASE == 1 ? a.panel1 : a.panel2);
    int* queues = PHASE == 1 ? a.queues1 : a.g2.queues;
    const int my_xcd = blockIdx.x & 7;

    // Slab layout: row-major, 16-byte chunk c of row r sits at position c ^ swz(r); swz(r) = (r >> 2) & 3 for 64-byte
    // rows and (r >> 1) & 7 for 128-byte rows (16 consecutive rows of a fragment read then cover all 64 banks).
    // One copy instruction of the workgroup deposits 8 KiB = RPC whole rows: thread t writes position t % (ROWB / 16)
    // of row t / (ROWB / 16), so it fetches the chunk that belongs there.
    const int row0_64 = tid >> 2, row0_128 = tid >> 3;
    const int kcg_64 = (tid & 3) ^ ((row0_64 >> 2) & 3), kcg_128 = (tid & 7) ^ ((row0_128 >> 1) & 7);
    const int wave_bytes = wave * 1024;
    int frag_off64[2], frag_off128[4];
#pragma unroll
    for (int u = 0; u < 2; ++u) frag_off64[u] = l31 * 64 + ((((u << 1) | lhi) ^ ((l31 >> 2) & 3)) << 4);
#pragma unroll
    for (int u = 0; u < 4; ++u) frag_off128[u] = l31 * 128 + ((((u << 1) | lhi) ^ ((l31 >> 1) & 7)) << 4);

    // thread 0 pulls tickets (own queue first, then the others).  A ticket names (block, unit); it is a tile only if
    // the unit is the first of the tile its block's class makes of it.
    auto fetch = [&](int first_k) __attribute__((always_inline)) {
        int q = my_xcd, blk = -1, unit = -1, cls = 0;
        int4 info = make_int4(0, 0, 0, 0);
        // 1 = a tile, 0 = no tile behind this ticket, -1 = queue exhausted
        auto look = [&](int k) __attribute__((always_inline)) -> int {
            const int st = geom.decode(q, k, blk, unit);
            if (st != 1) { blk = -1; return st; }
            // (a scalar load: the plan is read-only here, and a vector load's return would be counted behind the
            //  slab copies in flight)
            const __attribute__((address_space(4))) int* entry =
                (const __attribute__((address_space(4))) int*)a.plan + 4 * (PLAN_HDR + __builtin_amdgcn_readfirstlane(blk));
            info = make_int4(entry[0], entry[1], entry[2], entry[3]);
            cls = info.w;
            if ((unit & ((1 << cls) - 1)) == 0) return 1;
            blk = -1;
            return 0;
        };
        // the first look stands outside the loop: the wait for first_k then counts the copies issued since
        int st = look(first_k);
        for (int tries = 0; st != 1;) {
            if (st < 0) { if (++tries == 8) break; q = (q + 1) & 7; }
            st = look(atomicAdd(&queues[q], 1));
        }
        if (FUSED && PHASE == 2 && blk >= 0) {
            // The rows of h this tile reads are complete when every phase-1 tile of the row block has signalled.  Phase-1
            // tickets are all taken before the first phase-2 ticket, and a workgroup that holds a phase-1 ticket never
            // waits, so the wait ends; the bound on it only turns a defect into a flagged wrong result instead of a hang.
            const int need = a.f / 128;
            for (int spins = 0; __hip_atomic_load(&a.ready[blk], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < need; ++spins) {
                __builtin_amdgcn_s_sleep(32);                                           // about 2048 cycles
                if (spins > (1 << 20)) { atomicOr((int*)&a.plan[0].y, 1); break; }      // seconds: a defect, flagged in the plan header
            }
        }
        s_ticket[0] = blk; s_ticket[1] = blk >= 0 ? (unit >> cls) : 0; s_ticket[2] = cls;
        s_ticket[3] = info.x; s_ticket[4] = info.y; s_ticket[5] = info.z;      // the plan entry travels with the ticket
    };
    if (tid == 0) fetch(atomicAdd(&queues[my_xcd], 1));
    __syncthreads();
    if (s_ticket[0] < 0) return;

    // FUSED phase 1: the last two tiles of this workgroup whose completion has not been signalled yet (row block and
    // column units; block -1 = none).  A tile's output stores are the youngest memory operations when the next tile
    // begins, so waiting for them there would also wait for that tile's second slab; one tile later they are older
    // than everything the opening wait of a tile leaves outstanding (its second slab and the stores of the tile before
    // it) and are known to be complete at no extra cost.  So tile t is signalled when tile t + 2 opens, and what is left
    // when the workgroup runs out of tiles is signalled after a full wait.
    int sig_blk[2] = {-1, -1}, sig_units[2] = {0, 0};                // [0] = the tile before the previous one
    auto signal_ready = [&](int n) __attribute__((always_inline)) {
        // (every wavefront has passed the wait that covers these stores, and a barrier since)
#pragma unroll
        for (int i = 0; i < 2; ++i)
            if (i < n && tid == 0 && sig_blk[i] >= 0)
                __hip_atomic_fetch_add(&a.ready[sig_blk[i]], sig_units[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (n == 1) { sig_blk[0] = sig_blk[1]; sig_units[0] = sig_units[1]; sig_blk[1] = -1; }
        else        { sig_blk[0] = sig_blk[1] = -1; }
    };
    int cur_blk = 0;

    // ---- per-tile copy state: buffer resources and scalar offsets carry what is uniform, the per-thread byte offsets
    //      are fixed for a tile, so a copy costs no vector ALU work.  Rows past the end of the block re-read its last row.
    const __bf16* Abase = (PHASE == 1 ? a.x : a.g2.A);
    unsigned long long aB = 0;                         // address of the tile's first row of the A operand (plain rows)
    const unsigned char* a_ptr[GATHER ? 32 / NW : 1];        // address of this thread's chunk of each of its rows (gathered rows)
    // B rows come from w_gate / w_up (phase 1) or w_down (phase 2) of the tile's expert: base address of the first and
    // distance to the second.  (One variable per quantity, set once per tile: a choice between variables inside the
    // unrolled copy code would keep them in memory.)
    unsigned long long wB = 0, wB_up = 0;
    unsigned int b_voff = 0;
    bool counted_stores = false;                       // the previous tile's output went out as a known number of stores
    int m0 = 0, m_end = 0, nt = 0;
    unsigned int a_voff[32 / NW];
    unsigned int b_soff[8];

    auto setup = [&](auto tag, int nt_) __attribute__((always_inline)) {
        typedef Cls<decltype(tag)::value> C;
        nt = __builtin_amdgcn_readfirstlane(nt_);
        if (FUSED && PHASE == 1) cur_blk = __builtin_amdgcn_readfirstlane(s_ticket[0]);
        m0 = __builtin_amdgcn_readfirstlane(s_ticket[3]); m_end = __builtin_amdgcn_readfirstlane(s_ticket[4]);
        const int e = __builtin_amdgcn_readfirstlane(s_ticket[5]);
        const int rows = min(C::BMc, m_end - m0);
        const int row0 = C::ROWB == 128 ? row0_128 : row0_64, kcg = C::ROWB == 128 ? kcg_128 : kcg_64;
        int k0 = 0, r0 = 0;                                               // columns and rows of the operands the tile starts at
        if (PHASE == 2 && a.g2.etab) {
            const __attribute__((address_space(4))) int* t = (const __attribute__((address_space(4))) int*)a.g2.etab + 4 * e;
            k0 = t[0]; K = t[1]; r0 = t[2];
        }
        if constexpr (GATHER) {
#pragma unroll
            for (int i = 0; i < C::CA; ++i) {
                const int m = m0 + min(row0 + C::RPC * i, rows - 1);
                a_ptr[i] = (const unsigned char*)Abase + ((unsigned long long)(unsigned int)a.row_map[m] * (unsigned int)lda + kcg * 8) * 2ull;
            }
        } else {
            aB = (unsigned long long)Abase + ((unsigned long long)(unsigned int)(m0 - r0) * (unsigned int)lda + (unsigned int)k0) * 2ull;
#pragma unroll
            for (int i = 0; i < C::CA; ++i) a_voff[i] = (unsigned int)(min(row0 + C::RPC * i, rows - 1) * lda + kcg * 8) * 2u;
        }
        // the B rows of the tile: 64-bit base at the tile's first column unit, 32-bit offsets from there
        const int u0 = min(nt * C::U, NU - 1);
        if (PHASE == 1) {
            wB = (unsigned long long)((const __bf16*)a.wg + ((size_t)e * a.f + (size_t)u0 * 128) * ldb);
            wB_up = (unsigned long long)((const __bf16*)a.wu + ((size_t)e * a.f + (size_t)u0 * 128) * ldb) - wB;
        } else {
            wB = (unsigned long long)(a.g2.B + (size_t)e * a.g2.strideB + (size_t)u0 * 256 * ldb + k0);
            wB_up = 0;
        }
        b_voff = (unsigned int)(row0 * ldb + kcg * 8) * 2u;
        constexpr int CPSTRIP = 128 / C::RPC;                             // copies per 128-row strip of the B slab
#pragma unroll
        for (int j = 0; j < C::CB; ++j) {
            const int strip = j / CPSTRIP;
            const int ug = min(nt * C::U + (strip >> 1), NU - 1) - u0;
            const int strip_row = PHASE == 1 ? ug * 128 : ug * 256 + (strip & 1) * 128;   // row from the tile's first B row
            b_soff[j] = (unsigned int)(strip_row + (j % CPSTRIP) * C::RPC) * (unsigned int)ldb * 2u;
        }
    };
    // copy n of slab s into slab buffer sbuf
    auto issue_copy = [&](auto tag, int s, int sbuf, int n) __attribute__((always_inline)) {
        typedef Cls<decltype(tag)::value> C;
        constexpr int CPSTRIP = 128 / C::RPC;
        unsigned char* base = smem + sbuf * C::SLAB + wave_bytes;
        const int koff = s * C::ROWB;                           // (plain locals: the builtin's operands must not be dependent expressions)
        if (n < C::CA) {
            if constexpr (GATHER) {
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(a_ptr[n] + koff),
                                                 (__attribute__((address_space(3))) void*)(base + n * (NW * 1024)), 16, 0, 0);
            } else {
                const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc((void*)aB, 0, 0xFFFFFFFF, 0x00020000);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsA, (__attribute__((address_space(3))) void*)(base + n * (NW * 1024)), 16,
                                                         a_voff[n], koff, 0, FUSED && PHASE == 2 ? DEVICE_SCOPE : 0);
            }
        } else {
            const int j = n - C::CA;
            const unsigned long long up = (j / CPSTRIP) & 1;
            const __amdgpu_buffer_rsrc_t rsB = __builtin_amdgcn_make_buffer_rsrc((void*)(wB + up * wB_up), 0, 0xFFFFFFFF, 0x00020000);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsB,
                                                     (__attribute__((address_space(3))) void*)(base + C::A_BYTES + j * (NW * 1024)), 16,
                                                     b_voff, b_soff[j] + koff, 0, 0);
        }
    };
    // slabs [first, last) of the tile go out at once (the tile's opening; later slabs are spaced between the MFMAs)
    auto prologue = [&](auto tag, int first, int last) __attribute__((always_inline)) {
        typedef Cls<decltype(tag)::value> C;
        const int NS = K / (C::ROWB / 2);
#pragma unroll
        for (int s = 0; s < C::NSS; ++s)
            if (s >= first && s < last && s < NS) {
#pragma unroll
                for (int n = 0; n < C::NCOPY; ++n) issue_copy(tag, s, s, n);
            }
    };
    // Addresses of the tile and its first slabs, one per buffer (every K here has more slabs than there are buffers).
    auto start_tile = [&](int nt_, int cls) __attribute__((always_inline)) {
        if (cls == 0)      { setup(std::integral_constant<int, 0>{}, nt_); prologue(std::integral_constant<int, 0>{}, 0, 2); }
        else               { setup(std::integral_constant<int, 1>{}, nt_); prologue(std::integral_constant<int, 1>{}, 0, 3); }
    };

    // One tile of the class given by `tag`; its first slabs (one per buffer) are in flight.  Returns the class of the
    // next tile (whose first slabs it has issued: slab 0 in its last slabs or before its own read-out, the others
    // before the read-out) or -1.
    auto run_tile = [&](auto tag) __attribute__((always_inline)) -> int {
        typedef Cls<decltype(tag)::value> C;
        constexpr int MB = C::MB, NQ = C::NQ, NSS = C::NSS, SUB = C::SUB;
        constexpr int ROWB = C::ROWB, NMF = MB * NQ, NR = MB + NQ;
        constexpr int LPS = C::NCOPY;                                   // copies every wavefront issues per slab
        constexpr int NSTORE = MB * (PHASE == 1 ? 4 : 8) * (EPI == 1 ? 3 : 1);      // 1 KiB stores per wavefront and tile
        constexpr bool COUNTABLE = (NSS - 1) * C::NCOPY + NSTORE < 64;     // (the counter of memory operations in flight has 6 bits)
        static_assert((NSS - 1) * C::NCOPY < 64 && NSS * C::SLAB <= STAGE_OFF, "pipeline shape");
        static_assert(Cls<0>::MB == Cls<1>::MB, "a tile of either class issues NSTORE output stores");
        const int NS = K / (ROWB / 2);
        const int wm = wave / C::WNW, wn = wave % C::WNW;
        const int b_wave_row = PHASE == 1 ? (wn >> 1) * 256 + (wn & 1) * 64 : wn * 128;
        auto bq = [](int q) { return PHASE == 1 ? (q >> 1) * 128 + (q & 1) * 32 : q * 32; };
        const unsigned char* fragA = smem + (wm * 32 * MB) * ROWB;
        const unsigned char* fragB = smem + C::A_BYTES + b_wave_row * ROWB;

        auto load_frag_one = [&](bf16x8 (&wf)[NQ], bf16x8 (&xf)[MB], int sbuf, int u, int i) __attribute__((always_inline)) {
            const int off = sbuf * C::SLAB + (ROWB == 128 ? frag_off128[u] : frag_off64[u & 1]);
            if (i < NQ) wf[i] = *reinterpret_cast<const bf16x8*>(fragB + off + bq(i) * ROWB);
            else        xf[i - NQ] = *reinterpret_cast<const bf16x8*>(fragA + off + (i - NQ) * 32 * ROWB);
        };
        auto wait_slabs = [&](int y) __attribute__((always_inline)) {
            if (y >= 2) wait_vmcnt<2 * LPS>(); else if (y == 1) wait_vmcnt<LPS>(); else wait_vmcnt<0>();
        };

        f32x16 acc[MB][NQ];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int q = 0; q < NQ; ++q)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mb][q][v] = 0.f;
        const int em0 = m0, em_end = m_end, ent = nt;                   // this tile's rows and column unit, for the read-out
        const int eblk = cur_blk;
        int nblk = -1, nnt = 0, ncls = 0;                                // ticket of the next tile
        bool chained = false;                                            // the next tile's slab 0 was issued inside this tile

        // Issued so far, oldest first: slab 0, the slabs of the other buffers, the previous tile's output stores.  The
        // stores need not be awaited when their number is known (memory operations of a wavefront are counted in order).
        if (COUNTABLE && counted_stores) wait_vmcnt<COUNTABLE ? (NSS - 1) * LPS + NSTORE : 0>(); else wait_vmcnt<(NSS - 1) * LPS>();
        lds_barrier();                   // slab 0 is in LDS
        if (FUSED && PHASE == 1) signal_ready(1);
        // Ticket of the next tile: the counter's old value returns while slab 0 is multiplied and is turned into a
        // ticket after that slab (waiting for it here would hold wavefront 0, and with it every barrier, until the
        // copies just issued have landed: memory operations of a wavefront return in order).
        int next_k = 0;
        if (tid == 0) next_k = atomicAdd(&queues[my_xcd], 1);
        bf16x8 wf[2][NQ], xf[2][MB];
#pragma unroll
        for (int i = 0; i < NR; ++i) load_frag_one(wf[0], xf[0], 0, 0, i);

        // Slab s in buffer buf.  NEW: slab s + NSS exists (its slot 0 follows this slab's barrier); OLD: slab s - 1 + NSS
        // exists (its later slots go out during this slab's K steps); FINAL: the tile's last slab.
        // CHAIN (256-row class followed by another tile of it): the next tile's slab 0 takes the place of "slab NS" --
        // 1: this is slab NS - 2; after its first K step no copy of this tile is left, the next tile's addresses are
        //    set up, and slot 0 of that slab 0 follows this slab's barrier;  2: this is slab NS - 1, slot 1 goes out.
        auto slab = [&](int s, int buf, auto new_tag, auto old_tag, auto final_tag, auto chain_tag) __attribute__((always_inline)) {
            constexpr bool NEW = decltype(new_tag)::value, OLD = decltype(old_tag)::value, FINAL = decltype(final_tag)::value;
            constexpr int CHAIN = decltype(chain_tag)::value;
            static_assert(CHAIN == 0 || (C::S2 == 0 && NSS == 2 && !NEW && (CHAIN == 1 ? OLD && !FINAL : !OLD && FINAL)), "chained slabs");
            const int nbuf = buf + 1 == NSS ? 0 : buf + 1;              // buffer of slab s + 1
            const int pbuf = buf == 0 ? NSS - 1 : buf - 1;              // buffer slab s - 1 has left
#pragma unroll
            for (int u = 0; u < SUB; ++u) {
                const int cur = u & 1, nxt = cur ^ 1;
                const bool last = u + 1 == SUB;
                // fragment reads of the next K step (from the next slab after the barrier) and this K step's share
                // of the copies alternate in program order, so that the scheduler may interleave them with the MFMAs
                int rbuf = buf, ru = u + 1;
                const bool reads = !(last && FINAL);
                if (last && !FINAL) {
                    if (NEW) wait_vmcnt<(NSS - 2) * LPS>(); else wait_slabs(min(NSS - 2, NS - 2 - s));
                    lds_barrier();
                    rbuf = nbuf; ru = 0;
                }
                const int n = last ? (NEW || CHAIN == 1 ? C::S0 : 0)
                                   : (CHAIN == 2 ? (u == 0 ? C::S1 : 0) : (!OLD ? 0 : (u == 0 ? C::S1 : (u == 1 ? C::S2 : 0))));
                const int c0 = last ? 0 : (u == 0 ? C::S0 : C::S0 + C::S1);
                const int cslab = (CHAIN == 1 && last) || CHAIN == 2 ? 0 : (last ? s + NSS : s - 1 + NSS);
                const int cbuf = last ? buf : pbuf;
#pragma unroll
                for (int i = 0; i < NMF; ++i) {
                    if (i < NR && reads) load_frag_one(wf[nxt], xf[nxt], rbuf, ru, i);
#pragma unroll
                    for (int j = (i * n + NMF - 1) / NMF; j < ((i + 1) * n + NMF - 1) / NMF; ++j) issue_copy(tag, cslab, cbuf, c0 + j);
                }
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int q = 0; q < NQ; ++q)
                        acc[mb][q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[cur][q], xf[cur][mb], acc[mb][q], 0, 0, 0);
#pragma unroll
                for (int i = 0; i < NMF; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                  // MFMA
                    if (i < NR) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                      // LDS read
#pragma unroll
                    for (int j = (i * n + NMF - 1) / NMF; j < ((i + 1) * n + NMF - 1) / NMF; ++j)
                        __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);                              // slab copy
                }
                __builtin_amdgcn_sched_barrier(0);
                if (CHAIN == 1 && u == 0) {                              // this tile's last copies are out
                    if (chained) setup(tag, nnt);                        // addresses of the next tile
                }
            }
        };
        {
            const std::true_type T{};
            const std::false_type F{};
            const std::integral_constant<int, 0> C0{};
            if constexpr (decltype(tag)::value == 0) {
                // 256-row class: K is a multiple of 128 and at least 256, so NS is even and >= 4; slab s sits in buffer s & 1
                slab(0, 0, T, F, F, C0);
                if (tid == 0) fetch(next_k);
                int s = 1;
                for (; s + 2 < NS; ++s) slab(s, s & 1, T, T, F, C0);
                // a barrier has passed since the next tile's ticket was written
                nblk = __builtin_amdgcn_readfirstlane(s_ticket[0]); nnt = __builtin_amdgcn_readfirstlane(s_ticket[1]);
                ncls = __builtin_amdgcn_readfirstlane(s_ticket[2]);
                chained = nblk >= 0 && ncls == 0 && !GATHER;
                // not chained: the two slots re-fetch this tile's slab 0 into the free buffer 0, which nobody reads
                slab(NS - 2, 0, F, T, F, std::integral_constant<int, 1>{});
                slab(NS - 1, 1, F, F, T, std::integral_constant<int, 2>{});
                if (!chained) wait_vmcnt<0>();                           // ... and is complete before buffer 0 is reused
            } else {
                int buf = 0;
                auto next = [&]() __attribute__((always_inline)) { buf = buf + 1 == NSS ? 0 : buf + 1; };
                if (NSS < NS) slab(0, 0, T, F, F, C0); else slab(0, 0, F, F, F, C0);        // (every K here has at least 2 slabs)
                next();
                if (tid == 0) fetch(next_k);
                int s = 1;
                for (; s + NSS < NS; ++s) { slab(s, buf, T, T, F, C0); next(); }
                if (s + 1 < NS && s - 1 + NSS < NS) { slab(s, buf, F, T, F, C0); next(); ++s; }
                for (; s + 1 < NS; ++s) { slab(s, buf, F, F, F, C0); next(); }
                slab(NS - 1, buf, F, F, T, C0);
            }
        }
        lds_barrier();                   // every fragment is in registers: all buffers are free; next ticket visible
        if (chained) {
            prologue(tag, 1, NSS);                                      // slab 0 is under way; the other buffers follow
        } else {
            nblk = __builtin_amdgcn_readfirstlane(s_ticket[0]); nnt = __builtin_amdgcn_readfirstlane(s_ticket[1]);
            ncls = __builtin_amdgcn_readfirstlane(s_ticket[2]);         // uniform: keeps the copy descriptors in scalar registers
            if (nblk >= 0) start_tile(nnt, ncls);                       // the next tile's first slabs fly during the epilogue
            lds_barrier();                                              // the ticket has been read: its bytes may stage output
        }

        // ---- epilogue.  acc[mb][q][v]: row l31 of row block mb; column 8*(v>>2) + 4*lhi + (v&3) of column block q.
        // A lane holds 4 consecutive columns of one row: stored from there, one instruction would touch 32 rows with
        // 16 bytes each, and the L2 takes one request per piece.  Each wavefront instead passes 32 rows x 64 columns at
        // a time through a private staging area in LDS (above the slab buffers, where the next tile is arriving) and
        // stores whole 128-byte lines: 16-byte chunk c of row r sits at position c ^ swz(r), conflict-free both ways.
        const int ug = ent * C::U + (wn >> 1);
        constexpr int SROW = 128;                                           // staged bytes per row: 64 columns
        constexpr int CPR = SROW / 16;                                      // chunks per row
        constexpr int RPI = 64 / CPR;                                       // rows one store instruction covers
        constexpr int NH = PHASE == 1 ? 1 : 2;                              // 64-column halves of the wavefront's output
        int lane_e = lane;
        asm volatile("" : "+v"(lane_e));                                    // address arithmetic stays here, not in registers held across the tile loop
        const int el31 = lane_e & 31, elhi = lane_e >> 5;
        const int sr = lane_e / CPR, sc = lane_e % CPR;
        auto swz = [](int r) { return (r >> 1) & 7; };
        unsigned char* stage = smem + STAGE_OFF + wave * STAGE_WAVE;
        unsigned char* wr = stage + el31 * SROW + elhi * 8;
        const int wrow = em0 + wm * 32 * MB;                                // first row of this wavefront
        const bool scatter = PHASE == 2 && (a.row_map || a.row_gate);
        // plain case: rows and columns past the end fall outside the buffer descriptor and are dropped, so every
        // wavefront issues exactly NSTORE stores per tile
        constexpr int NPASS = EPI == 1 ? 3 : 1;                             // outputs per tile: h, or dg, du and h
        const int live = ug < NU ? min(max(em_end - wrow, 0), 32 * MB) : 0;
        __amdgpu_buffer_rsrc_t rsO[NPASS];
        int rowb[NPASS];
#pragma unroll
        for (int pass = 0; pass < NPASS; ++pass) {
            __bf16* obase;
            if (PHASE == 2)                  { obase = a.g2.O + (long long)wrow * a.g2.ldo + ug * 256 + (wn & 1) * 128; rowb[pass] = a.g2.ldo * 2; }
            else if (EPI == 0 || pass == 2)  { obase = a.h + (long long)wrow * a.f + ug * 128 + (wn & 1) * 64; rowb[pass] = a.f * 2; }
            else                             { obase = a.dgu + (long long)wrow * (2 * a.f) + pass * a.f + ug * 128 + (wn & 1) * 64; rowb[pass] = a.f * 4; }
            const unsigned long long ob = (unsigned long long)obase;      // (made uniform explicitly: the descriptor must sit in scalar registers)
            const unsigned int ob_lo = (unsigned int)__builtin_amdgcn_readfirstlane((unsigned int)ob);       // (the builtin returns int:
            const unsigned int ob_hi = (unsigned int)__builtin_amdgcn_readfirstlane((unsigned int)(ob >> 32)); //  widen as unsigned)
            const unsigned long long ob_u = ((unsigned long long)ob_hi << 32) | ob_lo;
            rsO[pass] = __builtin_amdgcn_make_buffer_rsrc((void*)ob_u, 0, __builtin_amdgcn_readfirstlane(live * rowb[pass]), 0x00020000);
        }
        counted_stores = !scatter;
        if (!scatter || ug < NU) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                if (PHASE == 2 && scatter && a.row_gate) {                // router weight of the row
                    float gate = 1.0f;
                    if (wrow + mb * 32 + el31 < em_end) gate = a.row_gate[wrow + mb * 32 + el31];
#pragma unroll
                    for (int q = 0; q < NQ; ++q)
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc[mb][q][v] *= gate;
                }
                // backward pass: the gradient of the hidden activations at this lane's 2 x 4 groups of 4 columns (rows
                // and units past the end read the last valid ones; what is computed from them is not stored)
                // backward pass: the gradient of the hidden activations at this lane's 2 x 4 groups of 4 columns (rows
                // and units past the end read the last valid ones; what is computed from them is not stored)
                u32x2 dhv[EPI == 1 ? 8 : 1];
                if constexpr (EPI == 1) {
                    const int row_c = min(wrow + mb * 32 + el31, em_end - 1);
                    const __bf16* src = a.dh + (long long)row_c * a.lddh + min(ug, NU - 1) * 128 + (wn & 1) * 64 + elhi * 4;
#pragma unroll
                    for (int c = 0; c < 8; ++c) dhv[c] = *reinterpret_cast<const u32x2*>(src + c * 8);
                }
#pragma unroll
                for (int step = 0; step < NPASS; ++step) {
                // backward pass: h goes out first; the same sweep leaves dg and du in the accumulators of g and u, from
                // where the two later sweeps store them (one exponential per element)
                const int pass = EPI == 1 ? (step + 2) % 3 : 0;
#pragma unroll
                for (int hq = 0; hq < NH; ++hq) {
#pragma unroll
                    for (int q = 0; q < 2; ++q)
#pragma unroll
                        for (int vg = 0; vg < 4; ++vg) {
                            float hv[4];
                            if constexpr (EPI == 1) {
                                if (step == 0) {
                                    const bf16x4 d4 = __builtin_bit_cast(bf16x4, dhv[q * 4 + vg]);
#pragma unroll
                                    for (int j = 0; j < 4; ++j) {
                                        const float g = acc[mb][q][vg * 4 + j], u = acc[mb][q + 2][vg * 4 + j], dh = (float)d4[j];
                                        const float sig = __builtin_amdgcn_rcpf(1.0f + __expf(-g));
                                        hv[j] = (g * sig) * u;                                                  // h
                                        acc[mb][q][vg * 4 + j] = dh * u * (sig * (1.0f + g * (1.0f - sig)));    // dg = dh * u * silu'(g)
                                        acc[mb][q + 2][vg * 4 + j] = dh * (g * sig);                            // du = dh * silu(g)
                                    }
                                } else {
#pragma unroll
                                    for (int j = 0; j < 4; ++j) hv[j] = acc[mb][step == 1 ? q : q + 2][vg * 4 + j];
                                }
                            } else {
#pragma unroll
                                for (int j = 0; j < 4; ++j)
                                    hv[j] = PHASE == 1 ? silu(acc[mb][q][vg * 4 + j]) * acc[mb][q + 2][vg * 4 + j]
                                                       : acc[mb][hq * 2 + q][vg * 4 + j];
                            }
                            *reinterpret_cast<u32x2*>(wr + (((q * 4 + vg) ^ swz(el31)) << 4)) = pack4(hv[0], hv[1], hv[2], hv[3]);
                        }
                    u32x4 v[32 / RPI];
#pragma unroll
                    for (int i = 0; i < 32 / RPI; ++i) {
                        const int r = i * RPI + sr;
                        v[i] = *reinterpret_cast<const u32x4*>(stage + r * SROW + ((sc ^ swz(r)) << 4));
                    }
                    if (!scatter) {
#pragma unroll
                        for (int i = 0; i < 32 / RPI; ++i)
                            __builtin_amdgcn_raw_buffer_store_b128(v[i], rsO[pass], (mb * 32 + i * RPI + sr) * rowb[pass] + hq * SROW + sc * 16, 0,
                                                                   FUSED && PHASE == 1 ? DEVICE_SCOPE : 0);
                    } else {
#pragma unroll
                        for (int i = 0; i < 32 / RPI; ++i) {
                            const int m = wrow + mb * 32 + i * RPI + sr;
                            if (m < em_end)
                                *reinterpret_cast<u32x4*>(a.g2.O + (long long)mapped_row(a, m) * a.g2.ldo + ug * 256 + (wn & 1) * 128 + hq * 64 + sc * 8) = v[i];
                        }
                    }
                }
                }
                __builtin_amdgcn_sched_barrier(0);     // one row block at a time: keeps the accumulator read-out short-lived
            }
        }
        if (FUSED && PHASE == 1) { sig_blk[1] = eblk; sig_units[1] = min(C::U, NU - ent * C::U); }
        return nblk >= 0 ? ncls : -1;
    };

    int cls = __builtin_amdgcn_readfirstlane(s_ticket[2]);
    start_tile(__builtin_amdgcn_readfirstlane(s_ticket[1]), cls);
    while (cls >= 0) {
        if (cls == 0)      cls = run_tile(std::integral_constant<int, 0>{});
        else               cls = run_tile(std::integral_constant<int, 1>{});
    }
    if (FUSED && PHASE == 1) {           // the last two tiles of this workgroup
        wait_vmcnt<0>();
        lds_barrier();
        signal_ready(2);
    }
}

template <int PHASE, bool GATHER, int EPI = 0>
__global__ __launch_bounds__(NW * 64, 1)
void ffn_adaptive_kernel(FfnArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    ffn_adaptive_body<PHASE, GATHER, false, EPI>(a, smem);
}

// Both phases in one launch: a workgroup works through the phase-1 tiles until none is left to hand out, then
// through the phase-2 tiles, each of which starts when the rows of h it reads are complete (release by the writers,
// acquire by the reader, at device scope).  The tail of phase 1 is filled with phase-2 tiles, and a call costs one
// launch of the matrix kernels whatever the number of slices.
template <bool GATHER>
__global__ __launch_bounds__(NW * 64, 1)
void ffn_fused_kernel(FfnArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    ffn_adaptive_body<1, GATHER, true>(a, smem);
    __syncthreads();                     // the ticket area and the staging buffers change hands
    ffn_adaptive_body<2, false, true>(a, smem);
}

// Expands block-scaled E4M3 codes [rows][cols] to bf16, eight values per thread and step (HBM bound: 3 bytes per weight).
__global__ __launch_bounds__(256)
void ffn_expand_fp8_kernel(const unsigned char* __restrict__ codes, const float* __restrict__ scales, __bf16* __restrict__ out,
                           long long n8, int cols) {
    const int sc_cols = cols / 128;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += (long long)gridDim.x * blockDim.x) {
        const long long e = i * 8;                                     // 8 consecutive codes of one row (cols % 128 == 0)
        const long long row = e / cols;
        const int col = (int)(e - row * cols);
        const float scale = scales[(row / 128) * sc_cols + col / 128];
        const u32x2 c = *reinterpret_cast<const u32x2*>(codes + e);
        *reinterpret_cast<u32x4*>(out + e) = dequant8(c, scale);
    }
}

int plan_capacity(int M) { return M / 64 + MAX_GROUPS + 1; }
size_t h_bytes(int M, int f) { return (((size_t)M * f * 2) + 255) & ~(size_t)255; }
size_t ready_bytes(int M) { return (((size_t)plan_capacity(M) * sizeof(int)) + 255) & ~(size_t)255; }

std::atomic<int> g_force_rows{0};          // moe_ffn_tile_override: 0 = rows per tile chosen per call, else 64 / 128 / 256
std::atomic<int> g_force_kernels{0};       //                        1 = never the adaptive-shape kernels, 2 = adaptive-shape kernels, one launch per phase
std::atomic<int> g_force_panel{0};         //                        0 = panel width of the tile walk chosen per call, else column groups per panel
std::atomic<int> g_num_cus[64];            // compute units of device d (0 = not asked yet)
int num_cus() {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
    n = g_num_cus[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        g_num_cus[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

// Column groups per panel of the tile walk.  The walk sweeps a panel's weights once per row group; as long as one
// expert's weights of the phase (plus a row group's activations and results) fit the 256 MB memory-side cache with room
// to spare, one panel holds all column groups.  Beyond that every sweep would evict what the next one needs (a cyclic
// pattern just above an LRU cache's size misses every time), so the columns are split into panels of about 64 MB and
// the activations are streamed once per panel instead.
int panel_width(int units, size_t expert_weight_bytes, size_t unit_bytes) {
    const int ncg = (units + 7) / 8, cn = (units + ncg - 1) / ncg;
    if (expert_weight_bytes <= ((size_t)128 << 20)) return ncg;
    const size_t group_bytes = (size_t)cn * unit_bytes;
    const int w = (int)(((size_t)64 << 20) / (group_bytes ? group_bytes : 1));
    return w < 1 ? 1 : (w > ncg ? ncg : w);
}

// Tile shapes.  ROWS = rows per tile:
//   256: 8 wavefronts (4 x 2), 64 x 128 per wavefront, two 64-wide slabs of 64 KiB (whole cache lines per row; 1 workgroup per CU)
//   128: 4 wavefronts (2 x 2), 64 x 128 per wavefront, three 32-wide slabs of 24 KiB         (2 workgroups per CU)
//    64: 4 wavefronts (2 x 2), 32 x 128 per wavefront, three 32-wide slabs of 20 KiB         (2 workgroups per CU)
template <int ROWS> struct Shape;
template <> struct Shape<256> { static constexpr int WMW = 4, MB = 2, BK = 64, NST = 2, PER_CU = 1; };
template <> struct Shape<128> { static constexpr int WMW = 2, MB = 2, BK = 32, NST = 3, PER_CU = 2; };
template <> struct Shape<64>  { static constexpr int WMW = 2, MB = 1, BK = 32, NST = 3, PER_CU = 2; };

template <int PHASE, int ROWS, bool FP8>
moe_status launch_gemm(const FfnArgs& a, long long max_tiles, hipStream_t s) {
    typedef Shape<ROWS> S;
    constexpr size_t lds = (size_t)S::NST * (ROWS + BN) * S::BK * 2;
    static moe::DeviceOnce attr;
    auto kern = ffn_gemm_kernel<PHASE, S::WMW, S::MB, FP8, S::BK, S::NST, S::PER_CU>;
    int dev;
    if (attr.needed(dev)) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) { moe::note_hip_error(e, "hipFuncSetAttribute(MaxDynamicSharedMemorySize)"); return MOE_ERR_HIP; }
        attr.mark(dev);
    }
    const long long slots = (long long)num_cus() * S::PER_CU;
    const int grid = (int)(max_tiles < slots ? max_tiles : slots);
    moe::LaunchScope k(PHASE == 1 ? "ffn_gemm1_kernel" : "ffn_gemm2_kernel", s);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(S::WMW * 128), lds, s, a);
    return k.done();
}

template <int PHASE, bool GATHER, int EPI = 0>
moe_status launch_adaptive(const FfnArgs& a, long long max_tiles, hipStream_t s, const char* name = nullptr) {
    static moe::DeviceOnce attr;
    auto kern = ffn_adaptive_kernel<PHASE, GATHER, EPI>;
    int dev;
    if (attr.needed(dev)) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, ADAPTIVE_LDS);
        if (e != hipSuccess) { moe::note_hip_error(e, "hipFuncSetAttribute(MaxDynamicSharedMemorySize)"); return MOE_ERR_HIP; }
        attr.mark(dev);
    }
    const long long slots = num_cus();
    const int grid = (int)(max_tiles < slots ? max_tiles : slots);
    moe::LaunchScope k(name ? name : (PHASE == 1 ? "ffn_gemm1_kernel" : "ffn_gemm2_kernel"), s);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NW * 64), ADAPTIVE_LDS, s, a);
    return k.done();
}

template <bool GATHER>
moe_status launch_fused(const FfnArgs& a, long long max_tiles, hipStream_t s) {
    static moe::DeviceOnce attr;
    auto kern = ffn_fused_kernel<GATHER>;
    int dev;
    if (attr.needed(dev)) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, ADAPTIVE_LDS);
        if (e != hipSuccess) { moe::note_hip_error(e, "hipFuncSetAttribute(MaxDynamicSharedMemorySize)"); return MOE_ERR_HIP; }
        attr.mark(dev);
    }
    const long long slots = num_cus();
    const int grid = (int)(max_tiles < slots ? max_tiles : slots);
    moe::LaunchScope k("ffn_fused_kernel", s);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NW * 64), ADAPTIVE_LDS, s, a);
    return k.done();
}

moe_status launch_both_adaptive(const FfnArgs& a, long long max_blocks, hipStream_t s) {
    if (g_force_kernels.load(std::memory_order_relaxed) != 2) {
        const long long tiles = max_blocks * std::max(a.f / 128, a.d / 256);
        return a.row_map ? launch_fused<true>(a, tiles, s) : launch_fused<false>(a, tiles, s);
    }
    moe_status st = a.row_map ? launch_adaptive<1, true>(a, max_blocks * (a.f / 128), s)
                              : launch_adaptive<1, false>(a, max_blocks * (a.f / 128), s);
    if (st != MOE_OK) return st;
    return launch_adaptive<2, false>(a, max_blocks * (a.d / 256), s);
}

template <int ROWS, bool FP8>
moe_status launch_both(const FfnArgs& a, long long max_blocks, hipStream_t s) {
    moe_status st = launch_gemm<1, ROWS, FP8>(a, max_blocks * (a.f / 128), s);
    if (st != MOE_OK) return st;
    return launch_gemm<2, ROWS, FP8>(a, max_blocks * (a.d / BN), s);
}

// ---------------------------------------------------------------------------------- backward pass: helper kernels
constexpr int BWD_GEMMS = 6;                   // launches of the matrix kernels per backward call (each owns 8 queue counters)
constexpr int BWD_KPAD = 128, BWD_KMIN = 256;  // a K range is padded to whole pairs of 64-wide K slabs, four slabs at least
constexpr int BWD_MAX_SPLIT = 16;

// padded row count of an expert whose rows are contracted in P parts of equal length
__host__ __device__ inline int bwd_kpad(int rows, int P) {
    const int unit = BWD_KPAD * P;
    const int k = (rows + unit - 1) / unit * unit;
    return k < BWD_KMIN * P ? BWD_KMIN * P : k;
}

// Parts the contraction of a weight gradient is split into.  The gradients have few output tiles (E_loc * f / 256 row
// blocks times d / 256 column units) and a very long contraction (all rows of the expert): unsplit, a small layer does
// not fill the chip and a large one runs in a few coarse rounds.  Parts produce partial sums that are added in fp32.
int bwd_split(int M, int E_loc, int d, int f) {
    const long long tiles = (long long)E_loc * ((f + 255) / 256) * (d / 256);
    int P = 1;
    while (P < BWD_MAX_SPLIT && tiles * P < 8 * 256 && (long long)M / E_loc / (2 * P) >= 1024) P *= 2;
    return P;
}

// One workgroup.  Expert-major numbering of the schedule's rows (the weight gradients contract over all rows of an
// expert, which lie in one group per slice): expert e owns columns k0_e .. k0_e + K_e - 1 of the transposed operands,
// K_e = its row count padded as above; src_row[c] = schedule row behind column c, or -1 for padding.
// The contraction of expert e is split into P parts ("virtual experts" v = e * P + p with partial results of their own):
// etab[v] = (k0_e + p * K_e / P, K_e / P, v * f, 0).  Also clears the tile queue counters of the launches that follow.
__global__ __launch_bounds__(PLAN_THREADS)
void bwd_prep_kernel(const int32_t* __restrict__ offsets, int S, int e_loc, int M, int f, int cols_cap, int P, int4* __restrict__ etab,
                     int* __restrict__ src_row, int* __restrict__ counters, int32_t* __restrict__ w_offsets) {
    __shared__ int k0_of[MAX_GROUPS / 16];      // (e_loc <= 4096)
    const int tid = threadIdx.x;
    auto bound = [&](int g) { return min(max(offsets[g], 0), M); };
    for (int i = tid; i < cols_cap; i += PLAN_THREADS) src_row[i] = -1;
    for (int i = tid; i < BWD_GEMMS * 8; i += PLAN_THREADS) counters[i] = 0;
    for (int v = tid; v <= e_loc * P; v += PLAN_THREADS) w_offsets[v] = v * f;  // row groups of the weight gradients: f rows per part
    for (int e = tid; e < e_loc; e += PLAN_THREADS) {
        int rows = 0;
        for (int sl = 0; sl < S; ++sl) { const int g = sl * e_loc + e; rows += max(bound(g + 1) - bound(g), 0); }
        k0_of[e] = bwd_kpad(rows, P);
    }
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int e = 0; e < e_loc; ++e) {
            const int k = k0_of[e], kp = k / P;
            for (int p = 0; p < P; ++p) etab[e * P + p] = make_int4(run + p * kp, kp, (e * P + p) * f, 0);
            k0_of[e] = run;
            run += k;
        }
    }
    __syncthreads();
    // one wavefront per expert at a time walks its groups in slice order
    const int wave = tid >> 6, lane = tid & 63;
    for (int e = wave; e < e_loc; e += PLAN_THREADS / 64) {
        int base = k0_of[e];
        for (int sl = 0; sl < S; ++sl) {
            const int g = sl * e_loc + e;
            const int lo = bound(g), n = max(bound(g + 1) - lo, 0);
            for (int r = lane; r < n; r += 64)
                if (base + r < cols_cap) src_row[base + r] = lo + r;
            base += n;
        }
    }
}

// dst[c][col] (pitch ldd, c < C) = src[src_row[col]][c] (pitch lds_), zero where src_row[col] < 0: the rows of a
// row-major operand become the K-contiguous columns of its transpose, in expert-major order.  HBM bound.  64 x 64 tiles
// through LDS; both sides move 16 bytes per thread (C and lds_ are multiples of 8, cols and ldd of 64).
__global__ __launch_bounds__(256)
void bwd_gather_transpose_kernel(const __bf16* __restrict__ src, int lds_, int C, const int* __restrict__ src_row, int cols,
                                 __bf16* __restrict__ dst, long long ldd) {
    __shared__ unsigned short tile[64][72];                              // [feature][column], padded rows
    const int col0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
    const int part = threadIdx.x & 7, line = threadIdx.x >> 3;           // 8 threads per 64-value line, 32 lines per pass
    typedef unsigned short us8 __attribute__((ext_vector_type(8)));
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int r = line + 32 * p, col = col0 + r;
        const int m = col < cols ? src_row[col] : -1;
        us8 v = {0, 0, 0, 0, 0, 0, 0, 0};
        if (m >= 0 && c0 + part * 8 < C) v = *reinterpret_cast<const us8*>(reinterpret_cast<const unsigned short*>(src) + (size_t)m * lds_ + c0 + part * 8);
#pragma unroll
        for (int k = 0; k < 8; ++k) tile[part * 8 + k][r] = v[k];
    }
    __syncthreads();
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int c = c0 + line + 32 * p;
        if (c < C && col0 + part * 8 < cols)
            *reinterpret_cast<us8*>(reinterpret_cast<unsigned short*>(dst) + (size_t)c * ldd + col0 + part * 8) =
                *reinterpret_cast<const us8*>(&tile[line + 32 * p][part * 8]);
    }
}

// out[e][r] = sum over p of part[e * P + p][r] (n values per expert), added in fp32 in part order; 8 values per thread
__global__ __launch_bounds__(256)
void bwd_reduce_parts_kernel(const __bf16* __restrict__ part, int P, long long n, int E, __bf16* __restrict__ out) {
    typedef __attribute__((ext_vector_type(8))) __bf16 b8;
    const long long n8 = n / 8, total = n8 * E;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
        const long long e = i / n8, r = (i - e * n8) * 8;
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int p = 0; p < P; ++p) {
            const b8 v = *reinterpret_cast<const b8*>(part + ((e * P + p) * n + r));
#pragma unroll
            for (int k = 0; k < 8; ++k) acc[k] += (float)v[k];
        }
        b8 o;
#pragma unroll
        for (int k = 0; k < 8; ++k) o[k] = (__bf16)acc[k];
        *reinterpret_cast<b8*>(out + (e * n + r)) = o;
    }
}

__global__ void bwd_zero_kernel(unsigned int* __restrict__ p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

// Batched transpose: dst[b][c][coff + r] (pitch ldd, slices of dstride elements) = src[b][r][c] (R x C, contiguous);
// rows c in C .. Cpad-1 of dst are zero-filled over the same column range.
__global__ __launch_bounds__(256)
void bwd_transpose_kernel(const __bf16* __restrict__ src, int R, int C, int Cpad, __bf16* __restrict__ dst, long long ldd,
                          long long dstride, int coff) {
    __shared__ unsigned short tile[64][66];
    const int b = blockIdx.z;
    const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const unsigned short* s16 = reinterpret_cast<const unsigned short*>(src) + (size_t)b * R * C;
    for (int r = ty; r < 64; r += 4)
        tile[r][tx] = (r0 + r < R && c0 + tx < C) ? s16[(size_t)(r0 + r) * C + c0 + tx] : (unsigned short)0;
    __syncthreads();
    unsigned short* d16 = reinterpret_cast<unsigned short*>(dst) + (size_t)b * dstride;
    for (int r = ty; r < 64; r += 4) {
        const int c = c0 + r;
        if (c < Cpad && r0 + tx < R) d16[(size_t)c * ldd + coff + r0 + tx] = tile[tx][r];
    }
}

inline size_t al256(size_t b) { return (b + 255) & ~(size_t)255; }

struct BwdLayout {                              // byte offsets into the workspace of a backward call
    size_t plan_rows, ready_rows, plan_w, ready_w, counters, etab, w_offsets, src_row, wdt, wgut, dh, dgu, h, tx, tdy, th, tdg, tdu, dwdt, part, total;
    int f_pad, cols_cap, P;
};
BwdLayout bwd_layout(int M, int E_loc, int d, int f) {
    BwdLayout L;
    L.f_pad = (f + 255) / 256 * 256;
    L.P = bwd_split(M, E_loc, d, f);
    L.cols_cap = (M + BWD_KPAD - 1) / BWD_KPAD * BWD_KPAD + BWD_KMIN * L.P * E_loc;
    const int wrows = E_loc * L.P * f;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += al256(bytes); return at; };
    L.plan_rows = take((size_t)(plan_capacity(M) + PLAN_HDR) * sizeof(int4));
    L.ready_rows = take((size_t)plan_capacity(M) * sizeof(int));
    L.plan_w = take((size_t)(plan_capacity(wrows) + PLAN_HDR) * sizeof(int4));
    L.ready_w = take((size_t)plan_capacity(wrows) * sizeof(int));
    L.counters = take((size_t)BWD_GEMMS * 8 * sizeof(int));
    L.etab = take((size_t)E_loc * L.P * sizeof(int4));
    L.w_offsets = take((size_t)(E_loc * L.P + 1) * sizeof(int32_t));
    L.src_row = take((size_t)L.cols_cap * sizeof(int));
    L.wdt = take((size_t)E_loc * L.f_pad * d * 2);
    L.wgut = take((size_t)E_loc * d * 2 * f * 2);
    L.dh = take((size_t)M * L.f_pad * 2);
    L.dgu = take((size_t)M * 2 * f * 2);
    L.h = take((size_t)M * f * 2);
    L.tx = take((size_t)d * L.cols_cap * 2);
    L.tdy = take((size_t)d * L.cols_cap * 2);
    L.th = take((size_t)f * L.cols_cap * 2);
    L.tdg = take((size_t)f * L.cols_cap * 2);
    L.tdu = take((size_t)f * L.cols_cap * 2);
    L.dwdt = take((size_t)E_loc * f * d * 2);
    L.part = take(L.P > 1 ? (size_t)E_loc * L.P * f * d * 2 : 0);
    L.total = o;
    return L;
}

}  // namespace

extern "C" size_t moe_ffn_workspace_bytes(int M, int d, int f) {
    if (M < 0 || d < 1 || f < 1) return 0;
    return h_bytes(M, f) + (size_t)(plan_capacity(M) + PLAN_HDR) * sizeof(int4) + ready_bytes(M);
}

extern "C" moe_status moe_ffn_tile_override(int tile_rows, int kernels, int panel_groups) {
    if (tile_rows != 0 && tile_rows != 64 && tile_rows != 128 && tile_rows != 256) return MOE_ERR_INVALID_ARG;
    if (kernels < 0 || kernels > 2) return MOE_ERR_INVALID_ARG;
    if (panel_groups < 0) return MOE_ERR_INVALID_ARG;
    g_force_rows.store(tile_rows, std::memory_order_relaxed);
    g_force_kernels.store(kernels, std::memory_order_relaxed);
    g_force_panel.store(panel_groups, std::memory_order_relaxed);
    return MOE_OK;
}

extern "C" size_t moe_ffn_expanded_weights_bytes(int E_loc, int d, int f) {
    if (E_loc < 1 || d < 1 || f < 1) return 0;
    return (((size_t)3 * E_loc * d * f * 2) + 255) & ~(size_t)255;
}

extern "C" moe_status moe_expert_ffn_sliced_mapped(const void* x, const int32_t* offsets, int M, int S, int E_loc, int d, int f,
                                                   int weight_format, const void* w_gate, const void* w_up, const void* w_down,
                                                   const float* s_gate, const float* s_up, const float* s_down,
                                                   const int32_t* row_map, const float* row_gate, void* y,
                                                   void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (M < 0 || S < 0 || E_loc < 1 || d < 1 || f < 1 || !offsets) return MOE_ERR_INVALID_ARG;
    if (weight_format != MOE_W_BF16 && weight_format != MOE_W_FP8_E4M3_B128) return MOE_ERR_INVALID_ARG;
    if (!w_gate || !w_up || !w_down) return MOE_ERR_INVALID_ARG;
    const bool fp8 = weight_format == MOE_W_FP8_E4M3_B128;
    if (fp8 && (!s_gate || !s_up || !s_down)) return MOE_ERR_INVALID_ARG;
    if (d % 256 != 0 || f % 128 != 0) return MOE_ERR_UNSUPPORTED_SHAPE;
    const long long G = (long long)S * E_loc;
    if (G > MAX_GROUPS) return MOE_ERR_UNSUPPORTED_SHAPE;
    // (32-bit byte offsets inside one 256-row tile and inside one expert's matrices)
    if (d > (1 << 22) || f > (1 << 22) || (long long)d * f >= (1LL << 31)) return MOE_ERR_UNSUPPORTED_SHAPE;
    if (M == 0 || G == 0) return MOE_OK;
    if (!x || !y) return MOE_ERR_INVALID_ARG;
    // every operand is moved in 16-byte pieces
    if ((((uintptr_t)x | (uintptr_t)y | (uintptr_t)w_gate | (uintptr_t)w_up | (uintptr_t)w_down | (uintptr_t)workspace) & 15) != 0)
        return MOE_ERR_INVALID_ARG;
    const size_t base_bytes = moe_ffn_workspace_bytes(M, d, f);
    if (!workspace || workspace_bytes < base_bytes) return MOE_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;

    // fp8 weights and many rows per expert: the kernels that dequantise on the fly pay for it on every row block, so
    // when the caller has added room for it the weights are expanded to bf16 once per call (bit-identical values) and
    // the bf16 kernels run.  Worth it from about 2048 rows per expert on (3 bytes of traffic per weight against a
    // quarter of the time of 6 flop per weight and row).
    if (fp8 && (long long)M >= 2048LL * E_loc && workspace_bytes - base_bytes >= moe_ffn_expanded_weights_bytes(E_loc, d, f)) {
        __bf16* wg = (__bf16*)((char*)workspace + base_bytes);
        __bf16* wu = wg + (size_t)E_loc * f * d;
        __bf16* wd = wu + (size_t)E_loc * f * d;
        const long long n8 = (long long)E_loc * f * d / 8;
        const int blocks = (int)std::min<long long>((n8 + 255) / 256, 16LL * num_cus());
        moe::LaunchScope k("ffn_expand_fp8_kernel", s);
        // gate and up: [E_loc * f][d] with scales [E_loc * f / 128][d / 128]; down: [E_loc * d][f]
        hipLaunchKernelGGL(ffn_expand_fp8_kernel, dim3(blocks), dim3(256), 0, s, (const unsigned char*)w_gate, s_gate, wg, n8, d);
        hipLaunchKernelGGL(ffn_expand_fp8_kernel, dim3(blocks), dim3(256), 0, s, (const unsigned char*)w_up, s_up, wu, n8, d);
        hipLaunchKernelGGL(ffn_expand_fp8_kernel, dim3(blocks), dim3(256), 0, s, (const unsigned char*)w_down, s_down, wd, n8, f);
        moe_status st = k.done();
        if (st != MOE_OK) return st;
        return moe_expert_ffn_sliced_mapped(x, offsets, M, S, E_loc, d, f, MOE_W_BF16, wg, wu, wd, nullptr, nullptr, nullptr,
                                            row_map, row_gate, y, workspace, base_bytes, hip_stream);
    }

    // rows per tile: large groups take 256-row tiles, fragmented schedules smaller ones
    const long long avg = M / G;
    int bm = avg >= 768 ? 256 : (avg >= 96 ? 128 : 64);
    if (const int forced = g_force_rows.load(std::memory_order_relaxed)) bm = forced;

    FfnArgs a;
    a.x = (const __bf16*)x;
    a.h = (__bf16*)workspace;
    a.y = (__bf16*)y;
    a.wg = w_gate; a.wu = w_up; a.wd = w_down;
    a.sg = s_gate; a.su = s_up; a.sd = s_down;
    int4* plan = (int4*)((char*)workspace + h_bytes(M, f));
    a.plan = plan;
    a.ready = (int*)(plan + PLAN_HDR + plan_capacity(M));
    a.d = d; a.f = f;
    a.row_map = row_map; a.row_gate = row_gate;
    a.queues1 = (int*)(plan + 1);
    a.g2.A = a.h; a.g2.lda = f;
    a.g2.B = (const __bf16*)w_down; a.g2.ldb = f; a.g2.strideB = (long long)d * f;
    a.g2.O = a.y; a.g2.ldo = d;
    a.g2.K = f; a.g2.NU = d / 256;
    a.g2.etab = nullptr;
    a.g2.queues = (int*)(plan + 3);
    a.dh = nullptr; a.lddh = 0; a.dgu = nullptr;
    a.panel1 = panel_width(f / 128, (size_t)2 * d * f * 2, (size_t)256 * d * 2);
    a.panel2 = panel_width(d / 256, (size_t)d * f * 2, (size_t)256 * f * 2);
    if (const int forced = g_force_panel.load(std::memory_order_relaxed)) a.panel1 = a.panel2 = forced;
    {
        moe::LaunchScope k("ffn_plan_kernel", s);
        hipLaunchKernelGGL(ffn_plan_kernel, dim3(1), dim3(PLAN_THREADS), 0, s, offsets, (int)G, E_loc, M, bm,
                           plan_capacity(M), plan, a.ready);
        moe_status st = k.done();
        if (st != MOE_OK) return st;
    }
    const long long max_blocks = M / bm + G;
    // (the adaptive kernel chains tiles over their last two slabs: at least four 64-wide slabs, f >= 256; d always is)
    if (bm == 256 && !fp8 && f >= 256 && g_force_kernels.load(std::memory_order_relaxed) != 1) return launch_both_adaptive(a, max_blocks, s);
    if (fp8) {
        if (bm == 256) return launch_both<256, true>(a, max_blocks, s);
        if (bm == 128) return launch_both<128, true>(a, max_blocks, s);
        return launch_both<64, true>(a, max_blocks, s);
    }
    if (bm == 256) return launch_both<256, false>(a, max_blocks, s);
    if (bm == 128) return launch_both<128, false>(a, max_blocks, s);
    return launch_both<64, false>(a, max_blocks, s);
}

extern "C" moe_status moe_expert_ffn_sliced(const void* x, const int32_t* offsets, int M, int S, int E_loc, int d, int f,
                                            int weight_format, const void* w_gate, const void* w_up, const void* w_down,
                                            const float* s_gate, const float* s_up, const float* s_down, void* y,
                                            void* workspace, size_t workspace_bytes, void* hip_stream) {
    return moe_expert_ffn_sliced_mapped(x, offsets, M, S, E_loc, d, f, weight_format, w_gate, w_up, w_down, s_gate, s_up,
                                        s_down, nullptr, nullptr, y, workspace, workspace_bytes, hip_stream);
}

extern "C" size_t moe_ffn_backward_workspace_bytes(int M, int E_loc, int d, int f) {
    if (M < 0 || E_loc < 1 || d < 1 || f < 1) return 0;
    return bwd_layout(M, E_loc, d, f).total;
}

extern "C" moe_status moe_expert_ffn_backward_sliced(const void* x, const void* dy, const int32_t* offsets, int M, int S, int E_loc,
                                                     int d, int f, const void* w_gate, const void* w_up, const void* w_down,
                                                     void* dx, void* dw_gate, void* dw_up, void* dw_down, void* workspace,
                                                     size_t workspace_bytes, void* hip_stream) {
    if (M < 0 || S < 0 || E_loc < 1 || d < 1 || f < 1 || !offsets) return MOE_ERR_INVALID_ARG;
    if (!w_gate || !w_up || !w_down || !dw_gate || !dw_up || !dw_down) return MOE_ERR_INVALID_ARG;
    if (d % 256 != 0 || f % 128 != 0 || f < 256) return MOE_ERR_UNSUPPORTED_SHAPE;
    const long long G = (long long)S * E_loc;
    if (G > MAX_GROUPS || E_loc > MAX_GROUPS / 16 || (long long)E_loc * BWD_MAX_SPLIT * f >= (1LL << 31)) return MOE_ERR_UNSUPPORTED_SHAPE;
    if (d > (1 << 22) || f > (1 << 21) || (long long)d * f >= (1LL << 30)) return MOE_ERR_UNSUPPORTED_SHAPE;
    if (M > 0 && (!x || !dy || !dx)) return MOE_ERR_INVALID_ARG;
    if ((((uintptr_t)x | (uintptr_t)dy | (uintptr_t)dx | (uintptr_t)w_gate | (uintptr_t)w_up | (uintptr_t)w_down | (uintptr_t)dw_gate |
          (uintptr_t)dw_up | (uintptr_t)dw_down | (uintptr_t)workspace) & 15) != 0)
        return MOE_ERR_INVALID_ARG;
    const BwdLayout L = bwd_layout(M, E_loc, d, f);
    // 32-bit byte offsets inside one 256-row tile of the transposed operands (row pitch = cols_cap)
    if ((long long)L.cols_cap * 512 * 2 >= (1LL << 32)) return MOE_ERR_UNSUPPORTED_SHAPE;
    if (!workspace || workspace_bytes < L.total) return MOE_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    char* ws = (char*)workspace;
    int4* plan_rows = (int4*)(ws + L.plan_rows);
    int4* plan_w = (int4*)(ws + L.plan_w);
    int* counters = (int*)(ws + L.counters);
    int4* etab = (int4*)(ws + L.etab);
    int* src_row = (int*)(ws + L.src_row);
    __bf16 *wdt = (__bf16*)(ws + L.wdt), *wgut = (__bf16*)(ws + L.wgut), *dh = (__bf16*)(ws + L.dh), *dgu = (__bf16*)(ws + L.dgu);
    __bf16 *h = (__bf16*)(ws + L.h), *tx = (__bf16*)(ws + L.tx), *tdy = (__bf16*)(ws + L.tdy), *th = (__bf16*)(ws + L.th);
    __bf16 *tdg = (__bf16*)(ws + L.tdg), *tdu = (__bf16*)(ws + L.tdu), *dwdt = (__bf16*)(ws + L.dwdt);
    __bf16* part = (__bf16*)(ws + L.part);
    const int P = L.P, wrows = E_loc * P * f;
    moe_status st;

    // ---- plans (row blocks of the schedule; row blocks of the weight gradients: one group of f rows per expert),
    //      expert-major column numbering, transposed weights
    {
        moe::LaunchScope k("ffn_plan_kernel", s);
        hipLaunchKernelGGL(ffn_plan_kernel, dim3(1), dim3(PLAN_THREADS), 0, s, offsets, (int)G, E_loc, M, 256, plan_capacity(M), plan_rows,
                           (int*)(ws + L.ready_rows));
        if ((st = k.done()) != MOE_OK) return st;
    }
    {
        moe::LaunchScope k("bwd_prep_kernel", s);
        hipLaunchKernelGGL(bwd_prep_kernel, dim3(1), dim3(PLAN_THREADS), 0, s, offsets, S, E_loc, M, f, L.cols_cap, P, etab, src_row, counters,
                           (int32_t*)(ws + L.w_offsets));
        if ((st = k.done()) != MOE_OK) return st;
    }
    {
        moe::LaunchScope k("bwd_transpose_kernel", s);
        const dim3 blk(256);
        // w_down [E][d][f] -> wdt [E][f_pad][d] (rows f .. f_pad-1 zero)
        hipLaunchKernelGGL(bwd_transpose_kernel, dim3((d + 63) / 64, (L.f_pad + 63) / 64, E_loc), blk, 0, s, (const __bf16*)w_down, d, f,
                           L.f_pad, wdt, (long long)d, (long long)L.f_pad * d, 0);
        // w_gate, w_up [E][f][d] -> wgut [E][d][2f] = [gate^T | up^T]
        hipLaunchKernelGGL(bwd_transpose_kernel, dim3((f + 63) / 64, (d + 63) / 64, E_loc), blk, 0, s, (const __bf16*)w_gate, f, d, d, wgut,
                           (long long)2 * f, (long long)d * 2 * f, 0);
        hipLaunchKernelGGL(bwd_transpose_kernel, dim3((f + 63) / 64, (d + 63) / 64, E_loc), blk, 0, s, (const __bf16*)w_up, f, d, d, wgut,
                           (long long)2 * f, (long long)d * 2 * f, f);
        if ((st = k.done()) != MOE_OK) return st;
    }
    if (M == 0 || G == 0) {
        // no rows: the weight gradients are zero, dx is empty
        moe::LaunchScope k("bwd_zero_kernel", s);
        const size_t words = (size_t)E_loc * f * d / 2;
        for (void* p : {dw_gate, dw_up, dw_down}) hipLaunchKernelGGL(bwd_zero_kernel, dim3(1024), dim3(256), 0, s, (unsigned int*)p, words);
        return k.done();
    }

    FfnArgs a;
    a.x = (const __bf16*)x; a.h = h; a.y = nullptr;
    a.wg = w_gate; a.wu = w_up; a.wd = w_down;
    a.sg = a.su = a.sd = nullptr;
    a.plan = plan_rows;
    a.ready = (int*)(ws + L.ready_rows);
    a.d = d; a.f = f;
    a.row_map = nullptr; a.row_gate = nullptr;
    a.panel1 = a.panel2 = 1 << 20;
    a.dh = dh; a.lddh = L.f_pad; a.dgu = dgu;
    a.queues1 = counters + 8;
    a.g2.etab = nullptr;
    const long long row_blocks = M / 256 + G;

    // ---- dh = dy Wd: rows x f_pad, K = d
    a.g2.A = (const __bf16*)dy; a.g2.lda = d;
    a.g2.B = wdt; a.g2.ldb = d; a.g2.strideB = (long long)L.f_pad * d;
    a.g2.O = dh; a.g2.ldo = L.f_pad;
    a.g2.K = d; a.g2.NU = L.f_pad / 256;
    a.g2.queues = counters + 0;
    if ((st = launch_adaptive<2, false, 0>(a, row_blocks * a.g2.NU, s, "ffn_bwd_dh_kernel")) != MOE_OK) return st;
    // ---- g, u recomputed; dg, du, h
    if ((st = launch_adaptive<1, false, 1>(a, row_blocks * (f / 128), s, "ffn_bwd_act_kernel")) != MOE_OK) return st;
    // ---- dx = [dg | du] [Wg ; Wu]: rows x d, K = 2f
    a.g2.A = dgu; a.g2.lda = 2 * f;
    a.g2.B = wgut; a.g2.ldb = 2 * f; a.g2.strideB = (long long)d * 2 * f;
    a.g2.O = (__bf16*)dx; a.g2.ldo = d;
    a.g2.K = 2 * f; a.g2.NU = d / 256;
    a.g2.queues = counters + 16;
    if ((st = launch_adaptive<2, false, 0>(a, row_blocks * a.g2.NU, s, "ffn_bwd_dx_kernel")) != MOE_OK) return st;

    // ---- transposed, expert-major copies of the operands of the weight gradients
    {
        moe::LaunchScope k("bwd_gather_transpose_kernel", s);
        const int cb = (L.cols_cap + 63) / 64;
        hipLaunchKernelGGL(bwd_gather_transpose_kernel, dim3(cb, (d + 63) / 64), dim3(256), 0, s, (const __bf16*)x, d, d, src_row, L.cols_cap, tx, (long long)L.cols_cap);
        hipLaunchKernelGGL(bwd_gather_transpose_kernel, dim3(cb, (d + 63) / 64), dim3(256), 0, s, (const __bf16*)dy, d, d, src_row, L.cols_cap, tdy, (long long)L.cols_cap);
        hipLaunchKernelGGL(bwd_gather_transpose_kernel, dim3(cb, (f + 63) / 64), dim3(256), 0, s, (const __bf16*)h, f, f, src_row, L.cols_cap, th, (long long)L.cols_cap);
        hipLaunchKernelGGL(bwd_gather_transpose_kernel, dim3(cb, (f + 63) / 64), dim3(256), 0, s, (const __bf16*)dgu, 2 * f, f, src_row, L.cols_cap, tdg, (long long)L.cols_cap);
        hipLaunchKernelGGL(bwd_gather_transpose_kernel, dim3(cb, (f + 63) / 64), dim3(256), 0, s, (const __bf16*)dgu + f, 2 * f, f, src_row, L.cols_cap, tdu, (long long)L.cols_cap);
        if ((st = k.done()) != MOE_OK) return st;
    }
    // ---- weight gradients: one group of f rows per expert, K = the expert's (padded) row count
    {
        moe::LaunchScope k("ffn_plan_kernel", s);
        hipLaunchKernelGGL(ffn_plan_kernel, dim3(1), dim3(PLAN_THREADS), 0, s, (const int32_t*)(ws + L.w_offsets), E_loc * P, E_loc * P, wrows, 256,
                           plan_capacity(wrows), plan_w, (int*)(ws + L.ready_w));
        if ((st = k.done()) != MOE_OK) return st;
    }
    a.plan = plan_w;
    a.g2.etab = etab;
    a.g2.lda = L.cols_cap; a.g2.ldb = L.cols_cap; a.g2.strideB = 0;
    a.g2.ldo = d; a.g2.K = BWD_KMIN; a.g2.NU = d / 256;
    const long long w_blocks = wrows / 256 + E_loc * P;
    struct { const __bf16 *A, *B; __bf16* O; int q; const char* name; } wg[3] = {
        {tdg, tx, (__bf16*)dw_gate, 24, "ffn_bwd_dwg_kernel"}, {tdu, tx, (__bf16*)dw_up, 32, "ffn_bwd_dwu_kernel"}, {th, tdy, dwdt, 40, "ffn_bwd_dwd_kernel"}};
    for (int i = 0; i < 3; ++i) {
        a.g2.A = wg[i].A; a.g2.B = wg[i].B; a.g2.O = P > 1 ? part : wg[i].O; a.g2.queues = counters + wg[i].q;
        if ((st = launch_adaptive<2, false, 0>(a, w_blocks * a.g2.NU, s, wg[i].name)) != MOE_OK) return st;
        if (P > 1) {                                                     // partial sums of the P parts -> the gradient
            moe::LaunchScope k("bwd_reduce_parts_kernel", s);
            const long long n = (long long)f * d;
            const int blocks = (int)std::min<long long>((n / 8 * E_loc + 255) / 256, 8LL * num_cus());
            hipLaunchKernelGGL(bwd_reduce_parts_kernel, dim3(blocks), dim3(256), 0, s, part, P, n, E_loc, wg[i].O);
            if ((st = k.done()) != MOE_OK) return st;
        }
    }
    // dWd^T [E][f][d] -> dw_down [E][d][f]
    moe::LaunchScope k("bwd_transpose_kernel", s);
    hipLaunchKernelGGL(bwd_transpose_kernel, dim3((f + 63) / 64, (d + 63) / 64, E_loc), dim3(256), 0, s, dwdt, f, d, d, (__bf16*)dw_down,
                       (long long)f, (long long)d * f, 0);
    return k.done();
}

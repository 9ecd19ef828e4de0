// moe_expert_ffn_sliced: SwiGLU expert FFN over all (slice, expert) row groups of a schedule
// (Section 2.1 "compute"; Section 2.2: per-batch fixed overheads are what fragmenting
// decompositions pay, so all slices are issued by launches whose number does not depend on the
// number of matchings).
//
// Two grouped GEMMs on the bf16 MFMA units, each a persistent kernel looping over output tiles:
//   phase 1:  H = silu(X Wg^T) * (X Wu^T)     tile = BM rows x (128 gate + 128 up) columns
//   phase 2:  Y = H Wd^T                      tile = BM rows x 256 columns
// A tile never spans two (slice, expert) groups.  Both operands are K-contiguous, are staged
// global -> registers -> LDS in 64-wide K slabs (double buffered, XOR-swizzled 16-byte chunks)
// and read back as 16-byte MFMA fragments.  4 wavefronts = 2 (rows) x 2 (columns); the weights
// feed the MFMA "A" port so that each lane ends up with 4 consecutive output columns of one row
// and can store 8 bytes at a time.
#include "common.hpp"
#include <stdlib.h>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

constexpr int FFN_THREADS = 256;
constexpr int BK = 64;                 // K slab: 64 bf16 = 128 bytes = 8 chunks of 16 bytes per row
constexpr int BN = 256;                // tile columns (phase 1: 128 gate + 128 up)
constexpr int ROW_BYTES = BK * 2;
constexpr int PLAN_THREADS = 1024;
constexpr int MAX_GROUPS = 65536;

struct FfnArgs {
    const __bf16* x;                   // [M][d]
    __bf16* h;                         // [M][f]   workspace
    __bf16* y;                         // [M][d]
    const void *wg, *wu, *wd;          // bf16 or fp8 codes
    const float *sg, *su, *sd;         // block scales (fp8) or null
    const int4* plan;                  // plan[0].x = number of row blocks; plan[1 + i] = (row0, row_end, expert, group)
    int d, f;
};

// ---------------------------------------------------------------------------------- plan kernel
// Splits every group into row blocks of BM rows.  One workgroup.  Malformed offsets cannot make
// it write outside the table: boundaries are clamped to [0, M] and to non-decreasing order, and
// entries beyond `cap` are dropped.
__global__ __launch_bounds__(PLAN_THREADS)
void ffn_plan_kernel(const int32_t* __restrict__ offsets, int G, int e_loc, int M, int bm, int cap, int4* __restrict__ plan) {
    __shared__ int wave_tot[PLAN_THREADS / 64];
    __shared__ int running;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) running = 0;
    __syncthreads();
    for (int g0 = 0; g0 < G; g0 += PLAN_THREADS) {
        const int g = g0 + tid;
        int lo = 0, hi = 0;
        if (g < G) {
            lo = min(max(offsets[g], 0), M);
            hi = min(max(offsets[g + 1], lo), M);
        }
        const int nblk = (hi - lo + bm - 1) / bm;
        int incl = nblk;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            int o = __shfl_up(incl, off);
            if (lane >= off) incl += o;
        }
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        int base = running;
        for (int w = 0; w < wave; ++w) base += wave_tot[w];
        int start = base + incl - nblk;
        for (int k = 0; k < nblk; ++k)
            if (start + k < cap) plan[1 + start + k] = make_int4(lo + k * bm, hi, g % e_loc, g);
        __syncthreads();
        if (tid == PLAN_THREADS - 1) running = base + incl;
        __syncthreads();
    }
    if (tid == 0) plan[0] = make_int4(min(running, cap), 0, 0, 0);
}

// ---------------------------------------------------------------------------------- helpers
__device__ __forceinline__ float silu(float g) { return g / (1.0f + __expf(-g)); }

__device__ __forceinline__ u32x2 pack4(float a, float b, float c, float d) {
    bf16x4 v = {(__bf16)a, (__bf16)b, (__bf16)c, (__bf16)d};
    return __builtin_bit_cast(u32x2, v);
}

// OCP FP8 E4M3 code -> float (bias 7, subnormals at exponent field 0, no infinities).
__device__ __forceinline__ float e4m3_to_float(unsigned int c) {
    unsigned int sign = (c & 0x80u) << 24, e = (c >> 3) & 0xFu, m = c & 0x7u;
    float sub = (float)m * 0.001953125f;                                  // m * 2^-9
    float nor = __uint_as_float(((e + 120u) << 23) | (m << 20));
    float mag = e == 0 ? sub : nor;
    return __uint_as_float(__float_as_uint(mag) | sign);
}
// 8 consecutive fp8 codes (8 bytes) times one scale -> 8 bf16
__device__ __forceinline__ u32x4 dequant8(u32x2 codes, float scale) {
    float v[8];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        v[k] = e4m3_to_float((codes.x >> (8 * k)) & 0xFFu) * scale;
        v[4 + k] = e4m3_to_float((codes.y >> (8 * k)) & 0xFFu) * scale;
    }
    bf16x8 o = {(__bf16)v[0], (__bf16)v[1], (__bf16)v[2], (__bf16)v[3], (__bf16)v[4], (__bf16)v[5], (__bf16)v[6], (__bf16)v[7]};
    return __builtin_bit_cast(u32x4, o);
}

// ---------------------------------------------------------------------------------- GEMM kernel
// PHASE 1: A = x (K = d), B rows 0..127 = gate rows, 128..255 = up rows of the tile's 128 columns.
// PHASE 2: A = h (K = f), B rows = 256 rows of w_down.
// MB = row blocks of 32 per wavefront: BM = 64 * MB.   FP8 = weights are block-scaled E4M3 codes.
template <int PHASE, int MB, bool FP8>
__global__ __launch_bounds__(FFN_THREADS)
void ffn_gemm_kernel(FfnArgs a) {
    constexpr int BM = 64 * MB;
    constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES, STAGE = A_BYTES + B_BYTES;
    constexpr int CA = BM * 8 / FFN_THREADS;          // 16-byte chunks per thread, A slab
    constexpr int CB = BN * 8 / FFN_THREADS;          // B slab (= 8)
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l31 = lane & 31, lhi = lane >> 5;
    const int K = PHASE == 1 ? a.d : a.f;
    const int NT = PHASE == 1 ? a.f / 128 : a.d / BN;
    const int KT = K / BK;
    const long long total = (long long)a.plan[0].x * NT;

    // staging coordinates of this thread: chunk c = tid + i*256 -> row = row0 + 32*i, 16-byte column kc
    const int row0 = tid >> 3, kc = tid & 7;
    const int st_off = row0 * ROW_BYTES + ((kc ^ (row0 & 7)) << 4);
    // fragment coordinates: row l31 of a 32-row block, chunk (2*ks + lhi), swizzled by (row & 7)
    int frag_off[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) frag_off[ks] = l31 * ROW_BYTES + ((((ks << 1) | lhi) ^ (lane & 7)) << 4);
    int brow[4];                                       // first B-slab row of this wave's 4 column blocks
#pragma unroll
    for (int q = 0; q < 4; ++q) brow[q] = PHASE == 1 ? ((q >> 1) * 128 + wn * 64 + (q & 1) * 32) : (wn * 128 + q * 32);

    // workgroups of one XCD (blockIdx % 8) take neighbouring tiles so that they share slabs in its L2
    const int grid = gridDim.x;
    const int slot = (grid % 8 == 0) ? (int)(blockIdx.x % 8) * (grid / 8) + (int)(blockIdx.x / 8) : (int)blockIdx.x;

    for (long long item = slot; item < total; item += grid) {
        const int blk = (int)(item / NT), nt = (int)(item - (long long)blk * NT);
        const int4 info = a.plan[1 + blk];
        const int m0 = info.x, m_end = info.y, e = info.z;
        const int rows = min(BM, m_end - m0);

        // ---- per-tile global addressing; rows past the group's end re-read its last row.
        //      B slab row r = row0 + 32*i: only i selects gate / up / 128-row block, so each B address is a
        //      wave-uniform base plus one per-thread byte offset.
        const __bf16* Abase = (PHASE == 1 ? a.x : (const __bf16*)a.h);
        int a_off[CA];
#pragma unroll
        for (int i = 0; i < CA; ++i) a_off[i] = (m0 + min(row0 + 32 * i, rows - 1)) * K + kc * 8;
        constexpr int ESZ = FP8 ? 1 : 2;
        const unsigned int b_voff = (unsigned int)(row0 * K + kc * 8) * ESZ;
        const unsigned char* bbase[CB];
        const float* sbase[CB];
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            long long wrow;                                               // first weight row of this 32-row strip
            const void* w;
            if (PHASE == 1) { wrow = (long long)e * a.f + nt * 128 + 32 * (i & 3); w = (i < 4) ? a.wg : a.wu; }
            else            { wrow = (long long)e * a.d + nt * BN + 32 * i;        w = a.wd; }
            bbase[i] = (const unsigned char*)w + wrow * K * ESZ;
            if (FP8) {
                // scale row of the 128 x 128 block holding the strip
                if (PHASE == 1) sbase[i] = ((i < 4) ? a.sg : a.su) + ((long long)e * (a.f / 128) + nt) * (K / 128);
                else            sbase[i] = a.sd + ((long long)e * (a.d / 128) + nt * 2 + (i >> 2)) * (K / 128);
            } else {
                sbase[i] = nullptr;
            }
        }

        f32x16 acc[MB][4];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mb][q][v] = 0.f;

        u32x4 ra[CA], rb[CB];
        auto load_slab = [&](int kt) {
#pragma unroll
            for (int i = 0; i < CA; ++i) ra[i] = *reinterpret_cast<const u32x4*>(Abase + a_off[i] + kt * BK);
#pragma unroll
            for (int i = 0; i < CB; ++i) {
                const unsigned char* src = bbase[i] + (size_t)kt * BK * ESZ + b_voff;
                if (!FP8) {
                    rb[i] = *reinterpret_cast<const u32x4*>(src);
                } else {
                    u32x2 codes = *reinterpret_cast<const u32x2*>(src);
                    rb[i] = dequant8(codes, sbase[i][kt >> 1]);
                }
            }
        };
        auto store_slab = [&](int stage) {
            unsigned char* sa = smem + stage * STAGE;
            unsigned char* sb = sa + A_BYTES;
#pragma unroll
            for (int i = 0; i < CA; ++i) *reinterpret_cast<u32x4*>(sa + st_off + i * 32 * ROW_BYTES) = ra[i];
#pragma unroll
            for (int i = 0; i < CB; ++i) *reinterpret_cast<u32x4*>(sb + st_off + i * 32 * ROW_BYTES) = rb[i];
        };

        load_slab(0);
        __syncthreads();                 // previous tile's readers are done with stage 0
        store_slab(0);
        __syncthreads();
        for (int kt = 0; kt < KT; ++kt) {
            if (kt + 1 < KT) load_slab(kt + 1);
            const unsigned char* sa = smem + (kt & 1) * STAGE + (wm * (BM / 2)) * ROW_BYTES;
            const unsigned char* sb = smem + (kt & 1) * STAGE + A_BYTES;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                bf16x8 wf[4], xf[MB];
#pragma unroll
                for (int q = 0; q < 4; ++q) wf[q] = *reinterpret_cast<const bf16x8*>(sb + brow[q] * ROW_BYTES + frag_off[ks]);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) xf[mb] = *reinterpret_cast<const bf16x8*>(sa + mb * 32 * ROW_BYTES + frag_off[ks]);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        acc[mb][q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[q], xf[mb], acc[mb][q], 0, 0, 0);
            }
            if (kt + 1 < KT) store_slab((kt + 1) & 1);
            __syncthreads();
        }

        // ---- epilogue.  acc[mb][q][v]: row m = l31 of row block mb; column n = 8*(v>>2) + 4*lhi + (v&3)
        //      of column block q
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int m = m0 + wm * (BM / 2) + mb * 32 + l31;
            if (m >= m_end) continue;
            if (PHASE == 1) {
                __bf16* out = a.h + (long long)m * a.f + nt * 128 + wn * 64 + 4 * lhi;
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
                __bf16* out = a.y + (long long)m * a.d + nt * BN + wn * 128 + 4 * lhi;
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int vg = 0; vg < 4; ++vg)
                        *reinterpret_cast<u32x2*>(out + q * 32 + vg * 8) =
                            pack4(acc[mb][q][vg * 4], acc[mb][q][vg * 4 + 1], acc[mb][q][vg * 4 + 2], acc[mb][q][vg * 4 + 3]);
            }
        }
    }
}

int plan_capacity(int M) { return M / 64 + MAX_GROUPS + 1; }
size_t h_bytes(int M, int f) { return (((size_t)M * f * 2) + 255) & ~(size_t)255; }

int g_num_cus = 0;
int num_cus() {
    if (g_num_cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            g_num_cus = n;
        else
            g_num_cus = 256;
    }
    return g_num_cus;
}

template <int PHASE, int MB, bool FP8>
moe_status launch_gemm(const FfnArgs& a, int grid, hipStream_t s) {
    constexpr size_t lds = 2 * (size_t)(64 * MB + BN) * ROW_BYTES;
    static bool attr_done = false;
    auto kern = ffn_gemm_kernel<PHASE, MB, FP8>;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) { moe::note_hip_error(e, "hipFuncSetAttribute(MaxDynamicSharedMemorySize)"); return MOE_ERR_HIP; }
        attr_done = true;
    }
    moe::LaunchScope k(PHASE == 1 ? "ffn_gemm1_kernel" : "ffn_gemm2_kernel", s);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(FFN_THREADS), lds, s, a);
    return k.done();
}

template <int MB, bool FP8>
moe_status launch_both(const FfnArgs& a, int grid1, int grid2, hipStream_t s) {
    moe_status st = launch_gemm<1, MB, FP8>(a, grid1, s);
    if (st != MOE_OK) return st;
    return launch_gemm<2, MB, FP8>(a, grid2, s);
}

}  // namespace

extern "C" size_t moe_ffn_workspace_bytes(int M, int d, int f) {
    if (M < 0 || d < 1 || f < 1) return 0;
    return h_bytes(M, f) + (size_t)(plan_capacity(M) + 1) * sizeof(int4);
}

extern "C" moe_status moe_expert_ffn_sliced(const void* x, const int32_t* offsets, int M, int S, int E_loc, int d, int f,
                                            int weight_format, const void* w_gate, const void* w_up, const void* w_down,
                                            const float* s_gate, const float* s_up, const float* s_down, void* y,
                                            void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (M < 0 || S < 0 || E_loc < 1 || d < 1 || f < 1 || !offsets) return MOE_ERR_INVALID_ARG;
    if (weight_format != MOE_W_BF16 && weight_format != MOE_W_FP8_E4M3_B128) return MOE_ERR_INVALID_ARG;
    if (!w_gate || !w_up || !w_down) return MOE_ERR_INVALID_ARG;
    const bool fp8 = weight_format == MOE_W_FP8_E4M3_B128;
    if (fp8 && (!s_gate || !s_up || !s_down)) return MOE_ERR_INVALID_ARG;
    if (d % 256 != 0 || f % 128 != 0) return MOE_ERR_UNSUPPORTED_SHAPE;
    const long long G = (long long)S * E_loc;
    if (G > MAX_GROUPS) return MOE_ERR_UNSUPPORTED_SHAPE;
    if ((long long)M * (d > f ? d : f) >= (1LL << 31)) return MOE_ERR_UNSUPPORTED_SHAPE;
    if (M == 0 || G == 0) return MOE_OK;
    if (!x || !y) return MOE_ERR_INVALID_ARG;
    if (!workspace || workspace_bytes < moe_ffn_workspace_bytes(M, d, f)) return MOE_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;

    // rows per wavefront tile: large groups take 256-row tiles, fragmented schedules smaller ones
    const long long avg = M / G;
    int mb = avg >= 768 ? 4 : (avg >= 96 ? 2 : 1);
    if (const char* ov = getenv("MOE_FFN_ROWS")) {
        int v = atoi(ov);
        if (v == 64) mb = 1; else if (v == 128) mb = 2; else if (v == 256) mb = 4;
    }
    const int bm = 64 * mb;

    FfnArgs a;
    a.x = (const __bf16*)x;
    a.h = (__bf16*)workspace;
    a.y = (__bf16*)y;
    a.wg = w_gate; a.wu = w_up; a.wd = w_down;
    a.sg = s_gate; a.su = s_up; a.sd = s_down;
    int4* plan = (int4*)((char*)workspace + h_bytes(M, f));
    a.plan = plan;
    a.d = d; a.f = f;
    {
        moe::LaunchScope k("ffn_plan_kernel", s);
        hipLaunchKernelGGL(ffn_plan_kernel, dim3(1), dim3(PLAN_THREADS), 0, s, offsets, (int)G, E_loc, M, bm,
                           plan_capacity(M), plan);
        moe_status st = k.done();
        if (st != MOE_OK) return st;
    }
    const long long max_blocks = M / bm + G;
    const int cus = num_cus();
    long long t1 = max_blocks * (f / 128), t2 = max_blocks * (d / BN);
    const int grid1 = (int)(t1 < cus ? t1 : cus), grid2 = (int)(t2 < cus ? t2 : cus);
    if (fp8) {
        if (mb == 4) return launch_both<4, true>(a, grid1, grid2, s);
        if (mb == 2) return launch_both<2, true>(a, grid1, grid2, s);
        return launch_both<1, true>(a, grid1, grid2, s);
    }
    if (mb == 4) return launch_both<4, false>(a, grid1, grid2, s);
    if (mb == 2) return launch_both<2, false>(a, grid1, grid2, s);
    return launch_both<1, false>(a, grid1, grid2, s);
}

// moe_combine_topk_sum: the last step of dispatch -> compute -> combine (Section 2.1): once the expert results are
// back at the rank that owns the tokens, every token's output is the router-weighted sum of the results of its topk
// experts.  HBM bound: topk rows of d bf16 values are read per token and one is written, each exactly once.
// Workgroups of 256 threads each walk a share of the tokens for one 2048-column stretch; a thread owns 8 consecutive
// columns (16 bytes), issues the loads of all its slots before it adds (the bytes in flight per thread are what fills
// the memory pipeline) and accumulates in fp32 in slot order.  Result rows are read once by the whole grid, so the loads
// are non-temporal.
#include "common.hpp"
#include <algorithm>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 cb_bf16x8;
typedef __attribute__((ext_vector_type(4))) unsigned int cb_u32x4;
constexpr int CB_THREADS = 256;
constexpr int CB_COLS = CB_THREADS * 8;        // columns one workgroup covers

template <int TOPK>                            // 0 = any topk (a loop), else unrolled
__global__ __launch_bounds__(CB_THREADS)
void combine_kernel(const __bf16* __restrict__ y, const int32_t* __restrict__ row_of, const float* __restrict__ gate,
                    int T, int topk, int d, int R, __bf16* __restrict__ out) {
    const int col = blockIdx.y * CB_COLS + threadIdx.x * 8;
    if (col >= d) return;
    if constexpr (TOPK != 0) {
        // A workgroup walks tokens blockIdx.x, blockIdx.x + gridDim.x, ...; the row numbers and weights of the next token
        // are fetched while the rows of the current one are in flight (otherwise every token costs two dependent
        // round trips to memory).
        int rows[TOPK], nrows[TOPK];
        float w[TOPK], nw[TOPK];
        auto fetch_index = [&](int t, int (&r)[TOPK], float (&g)[TOPK]) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < TOPK; ++j) {
                r[j] = row_of[(size_t)t * TOPK + j];
                g[j] = gate ? gate[(size_t)t * TOPK + j] : 1.0f;
            }
        };
        int t = blockIdx.x;
        if (t < T) fetch_index(t, rows, w);
        while (t < T) {
            cb_u32x4 v[TOPK];
#pragma unroll
            for (int j = 0; j < TOPK; ++j) {
                const bool live = rows[j] >= 0 && rows[j] < R;                // a dropped assignment contributes nothing
                if (!live) w[j] = 0.0f;
                v[j] = cb_u32x4{0u, 0u, 0u, 0u};
                if (live) v[j] = __builtin_nontemporal_load(reinterpret_cast<const cb_u32x4*>(y + (size_t)rows[j] * d + col));
            }
            const int tn = t + gridDim.x;
            if (tn < T) fetch_index(tn, nrows, nw);
            float acc[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[c] = 0.f;
#pragma unroll
            for (int j = 0; j < TOPK; ++j) {
                const cb_bf16x8 b = __builtin_bit_cast(cb_bf16x8, v[j]);
#pragma unroll
                for (int c = 0; c < 8; ++c) acc[c] = __builtin_fmaf(w[j], (float)b[c], acc[c]);
            }
            cb_bf16x8 o;
#pragma unroll
            for (int c = 0; c < 8; ++c) o[c] = (__bf16)acc[c];
            __builtin_nontemporal_store(__builtin_bit_cast(cb_u32x4, o), reinterpret_cast<cb_u32x4*>(out + (size_t)t * d + col));
            t = tn;
#pragma unroll
            for (int j = 0; j < TOPK; ++j) { rows[j] = nrows[j]; w[j] = nw[j]; }
        }
    } else {
        for (int t = blockIdx.x; t < T; t += gridDim.x) {
            const int32_t* rows = row_of + (size_t)t * topk;
            const float* g = gate ? gate + (size_t)t * topk : nullptr;
            float acc[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[c] = 0.f;
            for (int j = 0; j < topk; ++j) {
                const int r = rows[j];
                if (r < 0 || r >= R) continue;
                const float w = g ? g[j] : 1.0f;
                const cb_bf16x8 b = __builtin_bit_cast(cb_bf16x8, __builtin_nontemporal_load(reinterpret_cast<const cb_u32x4*>(y + (size_t)r * d + col)));
#pragma unroll
                for (int c = 0; c < 8; ++c) acc[c] = __builtin_fmaf(w, (float)b[c], acc[c]);
            }
            cb_bf16x8 o;
#pragma unroll
            for (int c = 0; c < 8; ++c) o[c] = (__bf16)acc[c];
            __builtin_nontemporal_store(__builtin_bit_cast(cb_u32x4, o), reinterpret_cast<cb_u32x4*>(out + (size_t)t * d + col));
        }
    }
}

}  // namespace

extern "C" moe_status moe_combine_topk_sum(const void* y, const int32_t* row_of, const float* gate, int T, int topk, int d, int R,
                                           void* out, void* hip_stream) {
    if (T < 0 || topk < 1 || d < 1 || R < 0) return MOE_ERR_INVALID_ARG;
    if (d % 8 != 0 || T > 0x7FFFFFFF / topk) return MOE_ERR_UNSUPPORTED_SHAPE;
    if (T == 0) return MOE_OK;
    if (!row_of || !out || (R > 0 && !y)) return MOE_ERR_INVALID_ARG;
    if ((((uintptr_t)y | (uintptr_t)out) & 15) != 0) return MOE_ERR_INVALID_ARG;         // rows are moved in 16-byte pieces
    hipStream_t s = (hipStream_t)hip_stream;
    const unsigned ycols = (unsigned)((d + CB_COLS - 1) / CB_COLS);
    if (ycols > 65535u) return MOE_ERR_UNSUPPORTED_SHAPE;
    int cus = 256;
    {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    }
    // about eight workgroups per compute unit, each walking its share of the tokens
    const unsigned per_col = (unsigned)std::max(1, cus * 8 / (int)ycols);
    const dim3 grid(std::min<unsigned>((unsigned)T, per_col), ycols);
    moe::LaunchScope k("combine_kernel", s);
    const __bf16* yy = (const __bf16*)y;
    __bf16* oo = (__bf16*)out;
    switch (topk) {
        case 1: hipLaunchKernelGGL(combine_kernel<1>, grid, dim3(CB_THREADS), 0, s, yy, row_of, gate, T, topk, d, R, oo); break;
        case 2: hipLaunchKernelGGL(combine_kernel<2>, grid, dim3(CB_THREADS), 0, s, yy, row_of, gate, T, topk, d, R, oo); break;
        case 4: hipLaunchKernelGGL(combine_kernel<4>, grid, dim3(CB_THREADS), 0, s, yy, row_of, gate, T, topk, d, R, oo); break;
        case 6: hipLaunchKernelGGL(combine_kernel<6>, grid, dim3(CB_THREADS), 0, s, yy, row_of, gate, T, topk, d, R, oo); break;
        case 8: hipLaunchKernelGGL(combine_kernel<8>, grid, dim3(CB_THREADS), 0, s, yy, row_of, gate, T, topk, d, R, oo); break;
        default: hipLaunchKernelGGL(combine_kernel<0>, grid, dim3(CB_THREADS), 0, s, yy, row_of, gate, T, topk, d, R, oo); break;
    }
    return k.done();
}

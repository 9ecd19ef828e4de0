// moe_combine_topk_sum: the last step of dispatch -> compute -> combine (Section 2.1): once the expert results are
// back at the rank that owns the tokens, every token's output is the router-weighted sum of the results of its topk
// experts.  HBM bound: topk rows of d bf16 values are read per token and one is written, each exactly once.
// One workgroup of 256 threads per (token, 2048-column stretch); a thread owns 8 consecutive columns (16 bytes), issues
// the loads of all its slots before it adds (the bytes in flight per thread are what fills the memory pipeline) and
// accumulates in fp32 in slot order.  Result rows are read once by the whole grid, so the loads are non-temporal.
#include "common.hpp"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 cb_bf16x8;
typedef __attribute__((ext_vector_type(4))) unsigned int cb_u32x4;
constexpr int CB_THREADS = 256;
constexpr int CB_COLS = CB_THREADS * 8;        // columns one workgroup covers

template <int TOPK>                            // 0 = any topk (a loop), else unrolled
__global__ __launch_bounds__(CB_THREADS)
void combine_kernel(const __bf16* __restrict__ y, const int32_t* __restrict__ row_of, const float* __restrict__ gate,
                    int topk, int d, int R, __bf16* __restrict__ out) {
    const int t = blockIdx.x;
    const int col = blockIdx.y * CB_COLS + threadIdx.x * 8;
    if (col >= d) return;
    const int K = TOPK ? TOPK : topk;
    const int32_t* rows = row_of + (size_t)t * K;
    const float* g = gate ? gate + (size_t)t * K : nullptr;
    float acc[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] = 0.f;
    if constexpr (TOPK != 0) {
        cb_u32x4 v[TOPK];
        float w[TOPK];
#pragma unroll
        for (int j = 0; j < TOPK; ++j) {
            const int r = rows[j];
            const bool live = r >= 0 && r < R;                        // a dropped assignment contributes nothing
            w[j] = live ? (g ? g[j] : 1.0f) : 0.0f;
            v[j] = cb_u32x4{0u, 0u, 0u, 0u};
            if (live) v[j] = __builtin_nontemporal_load(reinterpret_cast<const cb_u32x4*>(y + (size_t)r * d + col));
        }
#pragma unroll
        for (int j = 0; j < TOPK; ++j) {
            const cb_bf16x8 b = __builtin_bit_cast(cb_bf16x8, v[j]);
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[c] = __builtin_fmaf(w[j], (float)b[c], acc[c]);
        }
    } else {
        for (int j = 0; j < K; ++j) {
            const int r = rows[j];
            if (r < 0 || r >= R) continue;
            const float w = g ? g[j] : 1.0f;
            const cb_bf16x8 b = __builtin_bit_cast(cb_bf16x8, __builtin_nontemporal_load(reinterpret_cast<const cb_u32x4*>(y + (size_t)r * d + col)));
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[c] = __builtin_fmaf(w, (float)b[c], acc[c]);
        }
    }
    cb_bf16x8 o;
#pragma unroll
    for (int c = 0; c < 8; ++c) o[c] = (__bf16)acc[c];
    __builtin_nontemporal_store(__builtin_bit_cast(cb_u32x4, o), reinterpret_cast<cb_u32x4*>(out + (size_t)t * d + col));
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
    const dim3 grid((unsigned)T, (unsigned)((d + CB_COLS - 1) / CB_COLS));
    if (grid.y > 65535u) return MOE_ERR_UNSUPPORTED_SHAPE;
    moe::LaunchScope k("combine_kernel", s);
    const __bf16* yy = (const __bf16*)y;
    __bf16* oo = (__bf16*)out;
    switch (topk) {
        case 1: hipLaunchKernelGGL(combine_kernel<1>, grid, dim3(CB_THREADS), 0, s, yy, row_of, gate, topk, d, R, oo); break;
        case 2: hipLaunchKernelGGL(combine_kernel<2>, grid, dim3(CB_THREADS), 0, s, yy, row_of, gate, topk, d, R, oo); break;
        case 4: hipLaunchKernelGGL(combine_kernel<4>, grid, dim3(CB_THREADS), 0, s, yy, row_of, gate, topk, d, R, oo); break;
        case 6: hipLaunchKernelGGL(combine_kernel<6>, grid, dim3(CB_THREADS), 0, s, yy, row_of, gate, topk, d, R, oo); break;
        case 8: hipLaunchKernelGGL(combine_kernel<8>, grid, dim3(CB_THREADS), 0, s, yy, row_of, gate, topk, d, R, oo); break;
        default: hipLaunchKernelGGL(combine_kernel<0>, grid, dim3(CB_THREADS), 0, s, yy, row_of, gate, topk, d, R, oo); break;
    }
    return k.done();
}

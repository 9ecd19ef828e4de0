// moe_probe_mfma_bf16: what the matrix cores of this chip sustain on the FFN's instruction when nothing else moves --
// the measured ceiling beside the published peak (which assumes the peak shader clock; under load the clock is set
// by the power limit and depends on how many operand bits toggle).
#include "common.hpp"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int PROBE_THREADS = 256;     // four wavefronts, one per SIMD

// Every wavefront keeps 4 + 4 operand fragments and 16 accumulators in registers and issues 16 independent
// v_mfma_f32_32x32x16_bf16 per iteration; no memory traffic inside the loop.
__global__ __launch_bounds__(PROBE_THREADS)
void mfma_probe_kernel(float* __restrict__ sink, int iters, int data) {
    bf16x8 a[4], b[4];
    unsigned int st = (blockIdx.x * PROBE_THREADS + threadIdx.x) * 2654435761u + 12345u;
    // sum of four uniforms, centred and scaled: close enough to N(0, 1) for the toggle rate of the operand bits
    auto rnd = [&]() {
        float u = 0.f;
        for (int q = 0; q < 4; ++q) { st = st * 1664525u + 1013904223u; u += (float)(st >> 8) * (1.0f / 16777216.0f); }
        return (u - 2.0f) * 1.7320508f;
    };
    const float scale = data ? 1.0f : 0.0f;
    for (int i = 0; i < 4; ++i)
        for (int k = 0; k < 8; ++k) { a[i][k] = (__bf16)(scale * rnd()); b[i][k] = (__bf16)(scale * 0.02f * rnd()); }
    f32x16 acc[16];
    for (int i = 0; i < 16; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i * 4 + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i * 4 + j], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 16; ++i) s += acc[i][0];
    sink[(size_t)blockIdx.x * PROBE_THREADS + threadIdx.x] = s;
}

}  // namespace

extern "C" moe_status moe_probe_mfma_bf16(int data, int iters, int workgroups, float* sink, void* hip_stream) {
    if ((data != 0 && data != 1) || iters < 1 || iters > (1 << 22) || workgroups < 1 || workgroups > 4096 || !sink) return MOE_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    moe::LaunchScope k("mfma_probe_kernel", s);
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(workgroups), dim3(PROBE_THREADS), 0, s, sink, iters, data);
    return k.done();
}

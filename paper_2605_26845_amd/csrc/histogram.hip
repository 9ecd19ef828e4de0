// moe_route_histogram: top-k router output -> per-rank traffic matrix (Section 2.1 dispatch,
// Section 3 communication matrix).  HBM-bound scan of the ids with per-wavefront LDS
// histograms; one or several workgroups per (layer, source rank).
#include "common.hpp"

namespace {

constexpr int HIST_THREADS = 512;
constexpr int HIST_WAVES = HIST_THREADS / MOE_WAVE;

__global__ void hist_zero_kernel(int32_t* __restrict__ a, size_t na, int32_t* __restrict__ b, size_t nb) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t x = i; x < na; x += stride) a[x] = 0;
    if (b) for (size_t x = i; x < nb; x += stride) b[x] = 0;
}

// grid = (chunks, L*N).  Each workgroup scans one contiguous chunk of one source rank's ids.
// LDS holds `copies` private histograms of E bins (one per wavefront when E is small, so that
// lanes of different wavefronts never contend for a hot expert's bin).
// direct != 0 (one chunk per source): results are stored; otherwise they are added atomically to
// outputs that were zeroed beforehand.
__global__ __launch_bounds__(HIST_THREADS)
void hist_kernel(const int32_t* __restrict__ ids, int per_src, int chunk_len, int N, int E, int e_loc,
                 int copies, int direct, int32_t* __restrict__ traffic, int32_t* __restrict__ counts) {
    extern __shared__ int32_t lds_hist[];
    const int tid = threadIdx.x;
    const int src = blockIdx.y;                       // flattened (layer, source)
    for (int x = tid; x < copies * E; x += HIST_THREADS) lds_hist[x] = 0;
    __syncthreads();

    int32_t* mine = lds_hist + ((tid / MOE_WAVE) % copies) * E;
    const int begin = blockIdx.x * chunk_len;
    const int end = min(per_src, begin + chunk_len);
    const int32_t* base = ids + (size_t)src * per_src;
    const bool vec_ok = ((((uintptr_t)(base + begin)) & 15) == 0);
    int pos = begin;
    if (vec_ok) {
        const int nvec = (end - begin) / 4;
        typedef int v4i __attribute__((ext_vector_type(4)));
        const v4i* v = reinterpret_cast<const v4i*>(base + begin);
        for (int x = tid; x < nvec; x += HIST_THREADS) {
            v4i q = __builtin_nontemporal_load(v + x);
            if ((unsigned)q.x < (unsigned)E) atomicAdd(&mine[q.x], 1);
            if ((unsigned)q.y < (unsigned)E) atomicAdd(&mine[q.y], 1);
            if ((unsigned)q.z < (unsigned)E) atomicAdd(&mine[q.z], 1);
            if ((unsigned)q.w < (unsigned)E) atomicAdd(&mine[q.w], 1);
        }
        pos = begin + nvec * 4;
    }
    for (int x = pos + tid; x < end; x += HIST_THREADS) {
        int e = base[x];
        if ((unsigned)e < (unsigned)E) atomicAdd(&mine[e], 1);
    }
    __syncthreads();

    // fold the private copies into copy 0 and emit the per-expert counts
    for (int e = tid; e < E; e += HIST_THREADS) {
        int c = 0;
        for (int k = 0; k < copies; ++k) c += lds_hist[k * E + e];
        lds_hist[e] = c;
        if (counts) {
            if (direct) counts[(size_t)src * E + e] = c;
            else if (c) atomicAdd(&counts[(size_t)src * E + e], c);
        }
    }
    __syncthreads();
    // traffic[src][q] = sum over the experts of rank q
    for (int q = tid; q < N; q += HIST_THREADS) {
        int c = 0;
        for (int k = 0; k < e_loc; ++k) c += lds_hist[q * e_loc + k];
        if (direct) traffic[(size_t)src * N + q] = c;
        else if (c) atomicAdd(&traffic[(size_t)src * N + q], c);
    }
}

}  // namespace

extern "C" moe_status moe_route_histogram(const int32_t* ids, int L, int N, int T, int topk, int E,
                                          int32_t* traffic, int32_t* expert_counts, void* hip_stream) {
    if (L < 0 || N < 1 || T < 0 || topk < 1 || E < 1 || !traffic) return MOE_ERR_INVALID_ARG;
    if (E % N != 0 || E > MOE_MAX_EXPERTS) return MOE_ERR_UNSUPPORTED_SHAPE;
    const long long total = (long long)L * N * T * topk;
    if (total >= (1LL << 31) || (long long)L * N > 65535) return MOE_ERR_UNSUPPORTED_SHAPE;
    if (total > 0 && !ids) return MOE_ERR_INVALID_ARG;
    if (L == 0) return MOE_OK;
    hipStream_t s = (hipStream_t)hip_stream;
    const int per_src = T * topk;
    const int sources = L * N;
    // enough workgroups to cover the chip a few times over, chunks of at least 16 Ki ids,
    // chunk boundaries on 16-byte multiples
    int chunks = 1;
    if (sources < 1024 && per_src > 16384) {
        chunks = (1024 + sources - 1) / sources;
        int max_chunks = (per_src + 16383) / 16384;
        if (chunks > max_chunks) chunks = max_chunks;
    }
    int chunk_len = (per_src + chunks - 1) / chunks;
    chunk_len = (chunk_len + 3) & ~3;
    if (chunk_len < 4) chunk_len = 4;
    chunks = per_src > 0 ? (per_src + chunk_len - 1) / chunk_len : 1;
    const int direct = chunks == 1;
    int copies = 4096 / E;
    if (copies < 1) copies = 1;
    if (copies > HIST_WAVES) copies = HIST_WAVES;

    if (!direct) {
        moe::LaunchScope z("hist_zero_kernel", s);
        size_t na = (size_t)sources * N, nb = expert_counts ? (size_t)sources * E : 0;
        int blocks = (int)((na + nb + 255) / 256);
        if (blocks > 1024) blocks = 1024;
        hipLaunchKernelGGL(hist_zero_kernel, dim3(blocks), dim3(256), 0, s, traffic, na, expert_counts, nb);
        moe_status st = z.done();
        if (st != MOE_OK) return st;
    }
    moe::LaunchScope k("hist_kernel", s);
    hipLaunchKernelGGL(hist_kernel, dim3(chunks, sources), dim3(HIST_THREADS), (size_t)copies * E * sizeof(int32_t), s,
                       ids, per_src, chunk_len, N, E, E / N, copies, direct, traffic, expert_counts);
    return k.done();
}

// moe_slice_table: which rows reach the receiving rank in which matching (Sections 2.2 / 4.1:
// one source per receiver per matching; experts start when a matching's batch has arrived).
// One workgroup per source rank: it lists the matchings in which that source is wired to the
// receiver together with the cumulative amount shipped, then walks the source's assignments in
// arrival order and drops each one destined to the receiver into its window.
#include "common.hpp"

namespace {

constexpr int ST_THREADS = 1024;
constexpr int ST_WAVES = ST_THREADS / MOE_WAVE;
constexpr int ST_ITEMS = 8;         // assignments one thread takes per pass of the walk
constexpr int WIN_CAP = 2048;      // windows of one source kept in LDS (more spill to the workspace)
constexpr int CNT_CAP = 8192;      // (window, expert) counters of one source kept in LDS

// Work area of moe_slice_table_static: device memory owned by the library instead of a caller's workspace.  Every
// GPU the library runs on holds its own copy at its own address (looked up once per device, see static_scratch()).
constexpr size_t SCRATCH_BYTES = MOE_SLICE_TABLE_STATIC_BYTES;
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

struct ScanSmem {
    int wave_cnt[ST_WAVES];
    unsigned long long wave_sum[ST_WAVES];
};

// Block-wide scan in thread order: exclusive count of `flag`, inclusive sum of `val`;
// `total_*` are the block totals.  Two barriers.
__device__ __forceinline__ void block_scan(ScanSmem& sm, bool flag, unsigned long long val, int tid, int& excl_cnt,
                                           unsigned long long& incl_sum, int& total_cnt, unsigned long long& total_sum) {
    const int lane = tid & 63, wave = tid >> 6;
    unsigned long long b = __ballot(flag);
    int wcnt_excl = __popcll(b & ((1ULL << lane) - 1ULL));
    unsigned long long run = val;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        unsigned long long o = __shfl_up(run, off);
        if (lane >= off) run += o;
    }
    if (lane == 63) { sm.wave_cnt[wave] = __popcll(b); sm.wave_sum[wave] = run; }
    __syncthreads();
    int cbase = 0, ctot = 0;
    unsigned long long sbase = 0, stot = 0;
#pragma unroll
    for (int w = 0; w < ST_WAVES; ++w) {
        int c = sm.wave_cnt[w];
        unsigned long long s = sm.wave_sum[w];
        if (w < wave) { cbase += c; sbase += s; }
        ctot += c; stot += s;
    }
    __syncthreads();
    excl_cnt = cbase + wcnt_excl;
    incl_sum = sbase + run;
    total_cnt = ctot;
    total_sum = stot;
}

// Block-wide exclusive scan of a small per-thread count, in thread order; `total` is the block total.  Two barriers.
__device__ __forceinline__ void block_scan_counts(ScanSmem& sm, int cnt, int tid, int& excl, int& total) {
    const int lane = tid & 63, wave = tid >> 6;
    int run = cnt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int o = __shfl_up(run, off);
        if (lane >= off) run += o;
    }
    if (lane == 63) sm.wave_cnt[wave] = run;
    __syncthreads();
    int cbase = 0, ctot = 0;
#pragma unroll
    for (int w = 0; w < ST_WAVES; ++w) {
        int c = sm.wave_cnt[w];
        if (w < wave) cbase += c;
        ctot += c;
    }
    __syncthreads();
    excl = cbase + run - cnt;
    total = ctot;
}

__global__ void st_zero_kernel(int32_t* __restrict__ sizes, int G) {
    for (int x = blockIdx.x * blockDim.x + threadIdx.x; x < G; x += gridDim.x * blockDim.x) sizes[x] = 0;
}

__global__ __launch_bounds__(ST_THREADS)
void st_count_kernel(const int32_t* __restrict__ ids, int N, int per_src, int E, int e_loc, int r,
                     const int32_t* __restrict__ traffic, const uint8_t* __restrict__ perms,
                     const int32_t* __restrict__ durations, const int32_t* __restrict__ count_ptr, int kmax,
                     int32_t* __restrict__ sizes, int2* __restrict__ win_ws, int32_t* __restrict__ wcnt_ws,
                     int32_t* __restrict__ res_cnt, int32_t* __restrict__ wcount, int32_t* __restrict__ src_sizes) {
    // src_sizes (or null): [N][(kmax+2)*e_loc], this source's own count for every (slice, expert), written in full --
    // then `sizes` is not touched, nothing has to be zeroed beforehand and no global atomic is needed (requires
    // (kmax+1)*e_loc <= CNT_CAP, so that the counters of every source are in LDS)
    // wcnt_ws / res_cnt / wcount (all or none; only with (kmax+1)*e_loc <= CNT_CAP): per source the counts per
    // (window, expert), the counts of what was not shipped, and the number of windows -- what st_place_kernel needs
    __shared__ ScanSmem sm;
    __shared__ int2 lds_win[WIN_CAP];
    __shared__ int lds_cnt[CNT_CAP];
    const int tid = threadIdx.x;
    const int s = blockIdx.x;
    // the first pass of the walk below needs nothing of the schedule: its loads go out first and are in flight while
    // the windows are worked out (the kernel is a chain of dependent memory round trips otherwise)
    const int32_t* src = ids + (size_t)s * per_src;
    int e_first[ST_ITEMS];
#pragma unroll
    for (int k = 0; k < ST_ITEMS; ++k) e_first[k] = tid * ST_ITEMS + k < per_src ? src[tid * ST_ITEMS + k] : -1;
    int K = *count_ptr;
    K = K < 0 ? 0 : (K > kmax ? kmax : K);
    const long long amount = traffic[(size_t)s * N + r];
    int2* my_ws = win_ws + (size_t)s * kmax;

    // ---- windows of this source: (slice id, cumulative amount shipped up to and including it)
    int W = 0;
    if (s != r) {
        unsigned long long shipped = 0;
        for (int t0 = 0; t0 < K; t0 += ST_THREADS) {
            int t = t0 + tid;
            bool flag = t < K && perms[(size_t)t * N + s] == r;
            unsigned long long d = flag ? (unsigned long long)(unsigned int)max(durations[t], 0) : 0ULL;
            int excl, tot;
            unsigned long long incl, stot;
            block_scan(sm, flag, d, tid, excl, incl, tot, stot);
            if (flag) {
                unsigned long long cum = shipped + incl;
                if (cum > (unsigned long long)amount) cum = (unsigned long long)amount;
                int2 w2 = make_int2(1 + t, (int)cum);
                int idx = W + excl;
                my_ws[idx] = w2;
                if (idx < WIN_CAP) lds_win[idx] = w2;
            }
            W += tot;
            shipped += stot;
        }
    }
    const bool cnt_in_lds = (W + 1) * e_loc <= CNT_CAP;
    if (cnt_in_lds)
        for (int x = tid; x < (W + 1) * e_loc; x += ST_THREADS) lds_cnt[x] = 0;
    __threadfence_block();
    __syncthreads();
    const bool win_in_lds = W <= WIN_CAP;

    // ---- walk the assignments in arrival order, ST_ITEMS consecutive ones per thread and pass (one block scan per pass)
    int q_base = 0;
    const int e_lo = r * e_loc, e_hi = min(e_lo + e_loc, E);           // the receiver's experts
    for (int x0 = 0; x0 < per_src; x0 += ST_THREADS * ST_ITEMS) {
        const int first = x0 + tid * ST_ITEMS;
        int e[ST_ITEMS];
#pragma unroll
        for (int k = 0; k < ST_ITEMS; ++k) e[k] = x0 == 0 ? e_first[k] : (first + k < per_src ? src[first + k] : -1);
        int cnt = 0;
#pragma unroll
        for (int k = 0; k < ST_ITEMS; ++k) cnt += (e[k] >= e_lo && e[k] < e_hi) ? 1 : 0;
        int excl, tot;
        block_scan_counts(sm, cnt, tid, excl, tot);
        int q = q_base + excl;
#pragma unroll
        for (int k = 0; k < ST_ITEMS; ++k) {
            if (!(e[k] >= e_lo && e[k] < e_hi)) continue;
            // smallest window whose cumulative amount exceeds q; W means "not shipped"
            int lo = 0, hi = W;
            while (lo < hi) {
                int mid = (lo + hi) >> 1;
                int cum = win_in_lds ? lds_win[mid].y : my_ws[mid].y;
                if (cum > q) hi = mid; else lo = mid + 1;
            }
            const int el = e[k] - e_lo;
            if (cnt_in_lds) {
                atomicAdd(&lds_cnt[lo * e_loc + el], 1);
            } else {
                int slice = s == r ? 0 : (lo < W ? (win_in_lds ? lds_win[lo].x : my_ws[lo].x) : kmax + 1);
                atomicAdd(&sizes[(size_t)slice * e_loc + el], 1);
            }
            ++q;
        }
        q_base += tot;
    }
    if (cnt_in_lds) {
        __syncthreads();
        if (wcnt_ws) {
            int32_t* mine_ws = wcnt_ws + (size_t)s * (kmax + 1) * e_loc;
            for (int x = tid; x < (W + 1) * e_loc; x += ST_THREADS) mine_ws[x] = lds_cnt[x];
            if (tid < e_loc) res_cnt[(size_t)s * e_loc + tid] = s == r ? 0 : lds_cnt[W * e_loc + tid];
            if (tid == 0) wcount[s] = W;
        }
        if (src_sizes) {
            const int G = (kmax + 2) * e_loc;
            for (int x = tid; x < G; x += ST_THREADS) {
                const int slice = x / e_loc, el = x - slice * e_loc;
                int w = -1;                                     // window of this source that feeds the slice, if any
                if (s == r) {
                    w = slice == 0 ? 0 : -1;
                } else if (slice == kmax + 1) {
                    w = W;
                } else if (slice >= 1) {                        // windows are listed by ascending slice id
                    int lo = 0, hi = W;
                    while (lo < hi) {
                        int mid = (lo + hi) >> 1;
                        int id = win_in_lds ? lds_win[mid].x : my_ws[mid].x;
                        if (id < slice) lo = mid + 1; else hi = mid;
                    }
                    if (lo < W && (win_in_lds ? lds_win[lo].x : my_ws[lo].x) == slice) w = lo;
                }
                src_sizes[(size_t)s * G + x] = w >= 0 ? lds_cnt[w * e_loc + el] : 0;
            }
        } else {
            for (int x = tid; x < (W + 1) * e_loc; x += ST_THREADS) {
                int c = lds_cnt[x];
                if (c == 0) continue;
                int w = x / e_loc, el = x - w * e_loc;
                int slice = s == r ? 0 : (w < W ? (win_in_lds ? lds_win[w].x : my_ws[w].x) : kmax + 1);
                atomicAdd(&sizes[(size_t)slice * e_loc + el], c);
            }
        }
    }
}

// Row map of the receiving rank: for every row of the schedule (slice-major, then local expert, then source, then
// arrival order) its arrival index (position among the assignments destined to r, sources in rank order, each in
// its (token, slot) order) and its assignment index s * T * topk + t * topk + slot.  One workgroup per source walks
// the source's assignments as st_count_kernel did.  Windows are consecutive stretches of the arrival order, so the
// rank of an assignment inside its (window, expert) group is the number of earlier assignments of that expert minus
// those that fell into earlier windows; what no matching shipped is appended source by source.
constexpr int PLACE_MAX_ELOC = 64;
__global__ __launch_bounds__(ST_THREADS)
void st_place_kernel(const int32_t* __restrict__ ids, int N, int per_src, int E, int e_loc, int r,
                     const int32_t* __restrict__ traffic, int kmax, const int32_t* __restrict__ offsets,
                     const int2* __restrict__ win_ws, const int32_t* __restrict__ wcnt_ws, const int32_t* __restrict__ res_cnt,
                     const int32_t* __restrict__ wcount, int32_t* __restrict__ row_arrival, int32_t* __restrict__ row_assignment) {
    __shared__ ScanSmem sm;
    __shared__ int2 lds_win[WIN_CAP];
    __shared__ int pre[CNT_CAP];                       // assignments of expert el in windows before w, at [w * e_loc + el]
    __shared__ int cntw[ST_WAVES][PLACE_MAX_ELOC];     // this chunk: assignments of expert el seen by wavefront w
    __shared__ int run_el[PLACE_MAX_ELOC], res_base[PLACE_MAX_ELOC];
    __shared__ int src_base;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int s = blockIdx.x;
    const int W = wcount[s];
    const int2* my_ws = win_ws + (size_t)s * kmax;
    const bool win_in_lds = W <= WIN_CAP;
    for (int x = tid; x < W && x < WIN_CAP; x += ST_THREADS) lds_win[x] = my_ws[x];
    if (tid < e_loc) {
        const int32_t* c = wcnt_ws + (size_t)s * (kmax + 1) * e_loc;
        int acc = 0;
        for (int w = 0; w <= W; ++w) { pre[w * e_loc + tid] = acc; acc += c[w * e_loc + tid]; }
        int rb = 0;
        for (int s2 = 0; s2 < s; ++s2) rb += res_cnt[(size_t)s2 * e_loc + tid];
        res_base[tid] = rb;
        run_el[tid] = 0;
    }
    if (tid == 0) {
        int b = 0;
        for (int s2 = 0; s2 < s; ++s2) b += traffic[(size_t)s2 * N + r];
        src_base = b;
    }
    cntw[wave][lane] = 0;
    __syncthreads();

    int q_base = 0;
    const int32_t* src = ids + (size_t)s * per_src;
    for (int x0 = 0; x0 < per_src; x0 += ST_THREADS) {
        const int x = x0 + tid;
        const int e = x < per_src ? src[x] : -1;
        const bool mine = (unsigned)e < (unsigned)E && e / e_loc == r;
        int excl, tot;
        unsigned long long dummy_i, dummy_t;
        block_scan(sm, mine, 0ULL, tid, excl, dummy_i, tot, dummy_t);
        const int el = mine ? e % e_loc : 0;
        // rank among this wavefront's assignments of the same expert, and the wavefront's count per expert
        int rank_w = 0;
        unsigned long long todo = __ballot(mine);
        while (todo) {
            const int leader = __builtin_ctzll(todo);
            const int k = __builtin_amdgcn_readlane(el, leader);
            const unsigned long long peers = __ballot(mine && el == k);
            if (mine && el == k) rank_w = __popcll(peers & ((1ULL << lane) - 1ULL));
            if (lane == leader) cntw[wave][k] = __popcll(peers);
            todo &= ~peers;
        }
        __syncthreads();
        int before = 0;
        if (mine) {
            before = run_el[el] + rank_w;
            for (int w = 0; w < wave; ++w) before += cntw[w][el];
        }
        __syncthreads();
        if (tid < PLACE_MAX_ELOC) {
            int add = 0;
            for (int w = 0; w < ST_WAVES; ++w) { add += cntw[w][tid]; cntw[w][tid] = 0; }
            if (tid < e_loc) run_el[tid] += add;
        }
        if (mine) {
            const int q = q_base + excl;
            int lo = 0, hi = W;
            while (lo < hi) {
                int mid = (lo + hi) >> 1;
                int cum = win_in_lds ? lds_win[mid].y : my_ws[mid].y;
                if (cum > q) hi = mid; else lo = mid + 1;
            }
            const bool left = s != r && lo >= W;
            const int slice = s == r ? 0 : (left ? kmax + 1 : (win_in_lds ? lds_win[lo].x : my_ws[lo].x));
            const int pos = offsets[(size_t)slice * e_loc + el] + (left ? res_base[el] : 0) + before - pre[lo * e_loc + el];
            if (row_arrival) row_arrival[pos] = src_base + q;
            if (row_assignment) row_assignment[pos] = s * per_src + x;
        }
        q_base += tot;
        __syncthreads();
    }
}

// offsets[0] = 0, offsets[g+1] = sizes[0] + ... + sizes[g]; one workgroup.
__global__ __launch_bounds__(ST_THREADS)
void st_scan_kernel(const int32_t* __restrict__ sizes, int G, int32_t* __restrict__ offsets, const int32_t* __restrict__ src_sizes, int N) {
    // src_sizes != null: the size of group g is the sum of the N sources' own counts
    __shared__ ScanSmem sm;
    const int tid = threadIdx.x;
    unsigned long long base = 0;
    if (tid == 0) offsets[0] = 0;
    for (int g0 = 0; g0 < G; g0 += ST_THREADS) {
        int g = g0 + tid;
        unsigned long long v = 0ULL;
        if (g < G) {
            if (src_sizes) {
                for (int q = 0; q < N; ++q) v += (unsigned long long)src_sizes[(size_t)q * G + g];
            } else {
                v = (unsigned long long)sizes[g];
            }
        }
        int excl, tot;
        unsigned long long incl, stot;
        block_scan(sm, false, v, tid, excl, incl, tot, stot);
        if (g < G) offsets[g + 1] = (int32_t)(base + incl);
        base += stot;
    }
}

size_t sizes_bytes(int kmax, int e_loc) {
    size_t b = ((size_t)(kmax + 2) * e_loc) * sizeof(int32_t);
    return (b + 255) & ~(size_t)255;
}

// per-source sizes are used (and the zeroing kernel skipped) when every source's counters fit LDS and the table is small
bool dense_sizes(int N, int kmax, int e_loc) {
    return (long long)(kmax + 1) * e_loc <= CNT_CAP && (long long)N * (kmax + 2) * e_loc <= 65536;
}
size_t src_sizes_bytes(int N, int kmax, int e_loc) {
    return dense_sizes(N, kmax, e_loc) ? (((size_t)N * (kmax + 2) * e_loc * sizeof(int32_t)) + 255) & ~(size_t)255 : 0;
}

size_t win_bytes(int N, int kmax) { return (((size_t)N * (kmax > 0 ? kmax : 1) * sizeof(int2)) + 255) & ~(size_t)255; }

size_t rows_extra_bytes(int N, int kmax, int e_loc) {
    return ((size_t)N * (kmax + 1) * e_loc + (size_t)N * e_loc + (size_t)N) * sizeof(int32_t);
}

moe_status slice_table_impl(const int32_t* ids, int N, int T, int topk, int E, int r, const int32_t* traffic,
                            const uint8_t* perms, const int32_t* durations, const int32_t* count, int kmax,
                            int32_t* offsets, bool want_rows, int32_t* row_arrival, int32_t* row_assignment,
                            void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (N < 1 || T < 0 || topk < 1 || E < 1 || kmax < 0 || r < 0 || r >= N) return MOE_ERR_INVALID_ARG;
    if (!traffic || !count || !offsets || (kmax > 0 && (!perms || !durations))) return MOE_ERR_INVALID_ARG;
    if (E % N != 0 || N > 256) return MOE_ERR_UNSUPPORTED_SHAPE;
    const long long per_src = (long long)T * topk;
    if (per_src * N >= (1LL << 31)) return MOE_ERR_UNSUPPORTED_SHAPE;
    if (per_src > 0 && !ids) return MOE_ERR_INVALID_ARG;
    const int e_loc = E / N;
    const long long G = (long long)(kmax + 2) * e_loc;
    if (G >= (1LL << 30)) return MOE_ERR_UNSUPPORTED_SHAPE;
    if (want_rows && ((long long)(kmax + 1) * e_loc > CNT_CAP || e_loc > PLACE_MAX_ELOC)) return MOE_ERR_UNSUPPORTED_SHAPE;
    const size_t need = want_rows ? moe_slice_table_rows_workspace_bytes(N, kmax, E) : moe_slice_table_workspace_bytes(N, kmax, E);
    if (!workspace || workspace_bytes < need) return MOE_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    int32_t* sizes = (int32_t*)workspace;
    int2* win_ws = (int2*)((char*)workspace + sizes_bytes(kmax, e_loc));
    int32_t* src_sizes = dense_sizes(N, kmax, e_loc)
                             ? (int32_t*)((char*)workspace + sizes_bytes(kmax, e_loc) + win_bytes(N, kmax)) : nullptr;
    int32_t *wcnt_ws = nullptr, *res_cnt = nullptr, *wcount = nullptr;
    if (want_rows) {
        wcnt_ws = (int32_t*)((char*)workspace + moe_slice_table_workspace_bytes(N, kmax, E));
        res_cnt = wcnt_ws + (size_t)N * (kmax + 1) * e_loc;
        wcount = res_cnt + (size_t)N * e_loc;
    }
    if (!src_sizes) {
        moe::LaunchScope k("st_zero_kernel", s);
        int blocks = (int)((G + 255) / 256);
        if (blocks > 256) blocks = 256;
        hipLaunchKernelGGL(st_zero_kernel, dim3(blocks), dim3(256), 0, s, sizes, (int)G);
        moe_status st = k.done();
        if (st != MOE_OK) return st;
    }
    {
        moe::LaunchScope k("st_count_kernel", s);
        hipLaunchKernelGGL(st_count_kernel, dim3(N), dim3(ST_THREADS), 0, s, ids, N, (int)per_src, E, e_loc, r, traffic,
                           perms, durations, count, kmax, sizes, win_ws, wcnt_ws, res_cnt, wcount, src_sizes);
        moe_status st = k.done();
        if (st != MOE_OK) return st;
    }
    {
        moe::LaunchScope k("st_scan_kernel", s);
        hipLaunchKernelGGL(st_scan_kernel, dim3(1), dim3(ST_THREADS), 0, s, sizes, (int)G, offsets, src_sizes, N);
        moe_status st = k.done();
        if (st != MOE_OK || !want_rows) return st;
    }
    moe::LaunchScope k("st_place_kernel", s);
    hipLaunchKernelGGL(st_place_kernel, dim3(N), dim3(ST_THREADS), 0, s, ids, N, (int)per_src, E, e_loc, r, traffic, kmax,
                       offsets, win_ws, wcnt_ws, res_cnt, wcount, row_arrival, row_assignment);
    return k.done();
}

// Device address of `scratch` on the current device.  In host code the array's name is only a handle for the runtime,
// not a device address: the address is asked for once per device, with that device current, and kept.
std::atomic<void*> g_scratch_ptr[64];
moe_status static_scratch(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { moe::note_hip_error(e, "hipGetDevice"); return MOE_ERR_HIP; }
    if (dev < 0 || dev >= 64) return MOE_ERR_UNSUPPORTED_SHAPE;
    void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) { moe::note_hip_error(e, "hipGetSymbolAddress(scratch)"); return MOE_ERR_HIP; }
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return MOE_OK;
}

}  // namespace

extern "C" moe_status moe_slice_table_static(const int32_t* ids, int N, int T, int topk, int E, int r, const int32_t* traffic,
                                             const uint8_t* perms, const int32_t* durations, const int32_t* count, int kmax,
                                             int32_t* offsets, void* hip_stream) {
    if (N < 1 || kmax < 0 || E < 1) return MOE_ERR_INVALID_ARG;
    if (E % N != 0) return MOE_ERR_UNSUPPORTED_SHAPE;
    const size_t need = moe_slice_table_workspace_bytes(N, kmax, E);
    if (need == 0 || need > SCRATCH_BYTES) return MOE_ERR_WORKSPACE;      // the schedule is too long for the built-in work area
    void* ws = nullptr;
    moe_status st = static_scratch(&ws);
    if (st != MOE_OK) return st;
    // (nothing in the work area has to start at zero: the window lists are written before they are read, and the
    //  group sizes are either written in full by every source or cleared by the zeroing kernel of the sparse path)
    return slice_table_impl(ids, N, T, topk, E, r, traffic, perms, durations, count, kmax, offsets, false, nullptr, nullptr,
                            ws, SCRATCH_BYTES, hip_stream);
}

extern "C" size_t moe_slice_table_workspace_bytes(int N, int kmax, int E) {
    if (N < 1 || kmax < 0 || E < 1 || E % N != 0) return 0;
    return sizes_bytes(kmax, E / N) + win_bytes(N, kmax) + src_sizes_bytes(N, kmax, E / N);
}

extern "C" size_t moe_slice_table_rows_workspace_bytes(int N, int kmax, int E) {
    const size_t base = moe_slice_table_workspace_bytes(N, kmax, E);
    return base == 0 ? 0 : base + rows_extra_bytes(N, kmax, E / N);
}

extern "C" moe_status moe_slice_table(const int32_t* ids, int N, int T, int topk, int E, int r, const int32_t* traffic,
                                      const uint8_t* perms, const int32_t* durations, const int32_t* count, int kmax,
                                      int32_t* offsets, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return slice_table_impl(ids, N, T, topk, E, r, traffic, perms, durations, count, kmax, offsets, false, nullptr, nullptr,
                            workspace, workspace_bytes, hip_stream);
}

extern "C" moe_status moe_slice_table_rows(const int32_t* ids, int N, int T, int topk, int E, int r, const int32_t* traffic,
                                           const uint8_t* perms, const int32_t* durations, const int32_t* count, int kmax,
                                           int32_t* offsets, int32_t* row_arrival, int32_t* row_assignment, void* workspace,
                                           size_t workspace_bytes, void* hip_stream) {
    if (!row_arrival && !row_assignment) return MOE_ERR_INVALID_ARG;
    return slice_table_impl(ids, N, T, topk, E, r, traffic, perms, durations, count, kmax, offsets, true, row_arrival,
                            row_assignment, workspace, workspace_bytes, hip_stream);
}

// moe_decompose_greedy / moe_decompose_bvn: traffic matrix -> list of (permutation, duration).
//
// One 64-lane wavefront owns one matrix.  The residual (N x N int32, up to 64 KiB) lives in LDS;
// everything else (dual variables, matchings, adjacency bit masks) lives in registers, lane c
// holding column c (and column c+64 when N > 64) and, for row-indexed state, row c.  A single
// wavefront needs no barriers: cross-lane traffic is DPP reductions, ballots and readlane.
//
//   greedy (Section 3.2): maximum-weight perfect matching by shortest augmenting paths with
//     dual variables (the Jonker-Volgenant / Hungarian family the paper cites), duals kept warm
//     from one matching to the next (weights only ever decrease, so they stay feasible).
//   BvN (Section 3.1): integer padding to equal line sums, then perfect matchings inside the
//     support, repaired incrementally after every subtraction.
//   Both return the lexicographically smallest optimal permutation: the optimal permutations are
//     the perfect matchings of the tight graph (greedy) or of the support (BvN); rows are fixed
//     in order, each by one breadth-first search over alternating paths on 128-bit lane masks.
#include "common.hpp"
#include <limits.h>

namespace {

constexpr unsigned long long FNV_OFFSET = 14695981039346656037ULL;
constexpr unsigned long long FNV_PRIME = 1099511628211ULL;
constexpr int REDO_MARKED = 0x100;     // internal flag of greedy_kernel: decompose only the matrices marked NOT_DONE
constexpr int NOT_DONE = -1;           // counts[b] of a matrix the 16-bit pass could not hold

// ------------------------------------------------------------------------------ wave primitives
__device__ __forceinline__ int rdlane(int v, int l) {
    return __builtin_amdgcn_readlane(v, __builtin_amdgcn_readfirstlane(l));
}
template <int CTRL>
__device__ __forceinline__ int dpp(int v) {
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xF, 0xF, false);
}
// Minimum over the first 16 * NW lanes (NW = 1, 2, 4); the reduction inside a 16-lane row folds into the min instruction.
template <int CTRL>
__device__ __forceinline__ int min_dpp(int x) { return min(x, __builtin_amdgcn_mov_dpp(x, CTRL, 0xF, 0xF, true)); }
template <int CTRL>
__device__ __forceinline__ int max_dpp(int x) { return max(x, __builtin_amdgcn_mov_dpp(x, CTRL, 0xF, 0xF, true)); }
template <int NW>
__device__ __forceinline__ int wave_max_rows(int x) {
    x = max_dpp<0xB1>(x);
    x = max_dpp<0x4E>(x);
    x = max_dpp<0x141>(x);
    x = max_dpp<0x140>(x);
    int m = __builtin_amdgcn_readlane(x, 0);
    if (NW > 1) m = max(m, __builtin_amdgcn_readlane(x, 16));
    if (NW > 2) m = max(max(m, __builtin_amdgcn_readlane(x, 32)), __builtin_amdgcn_readlane(x, 48));
    return m;
}
template <int NW>
__device__ __forceinline__ int wave_min_rows(int x) {
    x = min_dpp<0xB1>(x);        // quad_perm [1,0,3,2]
    x = min_dpp<0x4E>(x);        // quad_perm [2,3,0,1]
    x = min_dpp<0x141>(x);       // row_half_mirror
    x = min_dpp<0x140>(x);       // row_mirror: every lane of a 16-lane row now holds the row's min
    int m = __builtin_amdgcn_readlane(x, 0);
    if (NW > 1) m = min(m, __builtin_amdgcn_readlane(x, 16));
    if (NW > 2) m = min(min(m, __builtin_amdgcn_readlane(x, 32)), __builtin_amdgcn_readlane(x, 48));
    return m;
}
// All 64 lanes must be active.
__device__ __forceinline__ int wave_min(int x) { return wave_min_rows<4>(x); }
__device__ __forceinline__ int wave_max(int x) { return wave_max_rows<4>(x); }
__device__ __forceinline__ int wave_sum(int x) {
    x += dpp<0xB1>(x);
    x += dpp<0x4E>(x);
    x += dpp<0x141>(x);
    x += dpp<0x140>(x);
    return __builtin_amdgcn_readlane(x, 0) + __builtin_amdgcn_readlane(x, 16) +
           __builtin_amdgcn_readlane(x, 32) + __builtin_amdgcn_readlane(x, 48);
}
// (the builtin takes the predicate as a lane mask; __ballot() takes an int, for which a predicate that already is a
//  lane mask goes through a vector register and a compare)
__device__ __forceinline__ unsigned long long ballot64(bool p) { return __builtin_amdgcn_ballot_w64(p); }
// The workgroup is a single wavefront, whose LDS accesses execute in program order: no barrier is needed
// between a lane's store and another lane's load, only that the compiler keeps that order and that pending
// LDS traffic has drained.  (__syncthreads() would also wait for every outstanding global store.)
__device__ __forceinline__ void lds_fence() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// lane-distributed arrays: element idx lives in lane idx & 63, slot idx >> 6 (one slot: 0 <= idx < 64, and an index
// outside that range matches no lane in set_at)
template <int NPL>
__device__ __forceinline__ int bcast(const int (&a)[NPL], int idx) {
    if constexpr (NPL == 1) return rdlane(a[0], idx);           // (the instruction takes the lane number modulo 64)
    int r = rdlane(a[0], idx & 63);
    if (NPL > 1) { int r1 = rdlane(a[NPL - 1], idx & 63); r = (idx >> 6) ? r1 : r; }
    return r;
}
template <int NPL>
__device__ __forceinline__ void set_at(int (&a)[NPL], int idx, int val, int lane) {
    if constexpr (NPL == 1) { if (lane == idx) a[0] = val; return; }
#pragma unroll
    for (int s = 0; s < NPL; ++s)
        if (lane == (idx & 63) && s == (idx >> 6)) a[s] = val;
}

// N-bit column/row sets as NPL 64-bit words
template <int NPL> struct Mask {
    unsigned long long w[NPL];
    __device__ __forceinline__ void clear() {
#pragma unroll
        for (int k = 0; k < NPL; ++k) w[k] = 0;
    }
    __device__ __forceinline__ bool any() const {
        unsigned long long o = 0;
#pragma unroll
        for (int k = 0; k < NPL; ++k) o |= w[k];
        return o != 0;
    }
    __device__ __forceinline__ bool test(int i) const {
        unsigned long long x = w[0];
        if (NPL > 1) x = (i >> 6) ? w[NPL - 1] : x;
        return (x >> (i & 63)) & 1ULL;
    }
    __device__ __forceinline__ void set(int i) {          // 0 <= i < 64 * NPL
        if constexpr (NPL == 1) { w[0] |= 1ULL << i; return; }
#pragma unroll
        for (int k = 0; k < NPL; ++k) if (k == (i >> 6)) w[k] |= 1ULL << (i & 63);
    }
    __device__ __forceinline__ void reset(int i) {
        if constexpr (NPL == 1) { w[0] &= ~(1ULL << i); return; }
#pragma unroll
        for (int k = 0; k < NPL; ++k) if (k == (i >> 6)) w[k] &= ~(1ULL << (i & 63));
    }
    __device__ __forceinline__ int first() const {        // index of the lowest set bit (any() must hold)
        int r = -1;
#pragma unroll
        for (int k = NPL - 1; k >= 0; --k) if (w[k]) r = 64 * k + __builtin_ctzll(w[k]);
        return r;
    }
};
template <int NPL>
__device__ __forceinline__ Mask<NPL> operator&(const Mask<NPL>& a, const Mask<NPL>& b) {
    Mask<NPL> r;
#pragma unroll
    for (int k = 0; k < NPL; ++k) r.w[k] = a.w[k] & b.w[k];
    return r;
}
// bits strictly below position i (SMALL: 0 <= i <= 32 is known)
template <int NPL, bool SMALL = false>
__device__ __forceinline__ Mask<NPL> below(int i) {
    Mask<NPL> r;
    if constexpr (SMALL) { r.w[0] = (1ULL << i) - 1ULL; return r; }
#pragma unroll
    for (int k = 0; k < NPL; ++k) {
        int rel = i - 64 * k;
        r.w[k] = rel <= 0 ? 0ULL : (rel >= 64 ? ~0ULL : ((1ULL << rel) - 1ULL));
    }
    return r;
}
// uniform copy of the mask held by row-lane `row`
template <int NPL>
__device__ __forceinline__ Mask<NPL> bcast_mask(const Mask<NPL> (&m)[NPL], int row) {
    Mask<NPL> r;
#pragma unroll
    for (int k = 0; k < NPL; ++k) {
        int lo[NPL], hi[NPL];
#pragma unroll
        for (int s = 0; s < NPL; ++s) { lo[s] = (int)(m[s].w[k] & 0xFFFFFFFFULL); hi[s] = (int)(m[s].w[k] >> 32); }
        unsigned int l = (unsigned int)bcast<NPL>(lo, row), h = (unsigned int)bcast<NPL>(hi, row);
        r.w[k] = ((unsigned long long)h << 32) | l;
    }
    return r;
}

// ------------------------------------------------------------------------------ shared pieces
// Copy one matrix into LDS (optionally with the diagonal forced to zero).
// 16-bit residual (the caller vouches for entries below 65536): returns false if an entry does not fit.
__device__ __forceinline__ bool load_matrix(const int32_t* __restrict__ A, uint16_t* R, int N, bool zero_diag, int lane) {
    const int total = N * N;
    bool ok = true;
    for (int x = lane; x < total; x += MOE_WAVE) {
        const int v = A[x];
        ok = ok && (unsigned)v < 65536u;
        R[x] = (uint16_t)v;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (zero_diag) {
        for (int i = lane; i < N; i += MOE_WAVE) R[i * N + i] = 0;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
    return __ballot(!ok) == 0;
}
__device__ __forceinline__ bool load_matrix(const int32_t* __restrict__ A, int32_t* R, int N, bool zero_diag, int lane) {
    const int total = N * N;
    if ((total & 3) == 0 && (((uintptr_t)A) & 15) == 0) {
        const int4* src = reinterpret_cast<const int4*>(A);
        int4* dst = reinterpret_cast<int4*>(R);
        for (int x = lane; x < total / 4; x += MOE_WAVE) dst[x] = src[x];
    } else {
        for (int x = lane; x < total; x += MOE_WAVE) R[x] = A[x];
    }
    lds_fence();
    if (zero_diag) {
        for (int i = lane; i < N; i += MOE_WAVE) R[i * N + i] = 0;
        lds_fence();
    }
    return true;
}
template <typename T>
__device__ __forceinline__ void store_matrix(const T* R, int32_t* __restrict__ out, int N, int lane) {
    const int total = N * N;
    for (int x = lane; x < total; x += MOE_WAVE) out[x] = R[x];
}

// Adjacency masks: row-lane r gets {j : pred(R[r][j], r, j)}; built row by row with ballots so
// that LDS reads are conflict free.
template <int NPL, typename T, typename Pred>
__device__ __forceinline__ void build_masks(const T* R, int N, int lane, Mask<NPL> (&tm)[NPL], Pred pred) {
#pragma unroll
    for (int s = 0; s < NPL; ++s) tm[s].clear();
    const Mask<NPL> cols = below<NPL>(N);
#pragma unroll 4
    for (int i = 0; i < N; ++i) {
        Mask<NPL> row;
#pragma unroll
        for (int s = 0; s < NPL; ++s) {
            int j = lane + 64 * s;
            row.w[s] = ballot64(pred(R[i * N + (j < N ? j : 0)], i, s)) & cols.w[s];
        }
#pragma unroll
        for (int s = 0; s < NPL; ++s)
            if (lane == (i & 63) && s == (i >> 6)) tm[s] = row;
    }
}

// One level of the alternating breadth-first search used by both the lexicographic pass and
// the BvN repair.  Rows of `open` (those that may still be visited) that touch a reached column are visited,
// leave `open` and remember that column; returns the set of rows visited in this level.  The sets of rows are
// uniform masks: a per-lane flag carried around the search loop would live in a vector register and cost a
// select and a compare per level.
// SMALL (N <= 32, here and below): the masks fit 32 bits and the per-lane arithmetic on them is done in 32 bits
// (64-bit shifts and compares run at a fraction of the 32-bit rate).
template <int NPL, bool SMALL = false>
__device__ __forceinline__ Mask<NPL> bfs_visit_rows(const Mask<NPL> (&tm)[NPL], const Mask<NPL>& reached, int lane,
                                                    Mask<NPL>& open, int (&parent)[NPL]) {
    Mask<NPL> vm;
    if constexpr (SMALL) {
        static_assert(NPL == 1, "32-bit masks");
        const unsigned int hit = (unsigned int)tm[0].w[0] & (unsigned int)reached.w[0];
        vm.w[0] = ballot64(hit != 0) & open.w[0];
        if (__builtin_amdgcn_inverse_ballot_w64(vm.w[0])) parent[0] = __builtin_ctz(hit);
        open.w[0] &= ~vm.w[0];
        return vm;
    }
#pragma unroll
    for (int s = 0; s < NPL; ++s) {
        Mask<NPL> hit = tm[s] & reached;
        vm.w[s] = ballot64(hit.any()) & open.w[s];
        if (__builtin_amdgcn_inverse_ballot_w64(vm.w[s])) parent[s] = hit.first();
        open.w[s] &= ~vm.w[s];
    }
    return vm;
}
// rows after row i (i = -1: all rows)
template <int NPL, bool SMALL = false>
__device__ __forceinline__ Mask<NPL> rows_after(int i, int N) {
    Mask<NPL> r = below<NPL, SMALL>(N), b = below<NPL, SMALL>(i + 1);
#pragma unroll
    for (int k = 0; k < NPL; ++k) r.w[k] &= ~b.w[k];
    return r;
}
// Columns whose current owner row is in `rows` join `reached`; `owned` = the columns that have an owner.
// (Every ballot here is fed by a single comparison and the sets are combined as uniform masks: a conjunction of
// per-lane conditions handed to a ballot is first turned into a 0/1 vector register and compared again.)
template <int NPL, bool SMALL = false>
__device__ __forceinline__ void bfs_reach_cols(const int (&p)[NPL], const Mask<NPL>& rows, const Mask<NPL>& owned, int lane,
                                               Mask<NPL>& reached) {
    if constexpr (SMALL) {
        reached.w[0] |= ballot64((((unsigned int)rows.w[0] >> (p[0] & 31)) & 1u) != 0) & owned.w[0];
        return;
    }
#pragma unroll
    for (int s = 0; s < NPL; ++s) reached.w[s] |= ballot64(rows.test(p[s] & (64 * NPL - 1))) & owned.w[s];
}
// Re-route along the parents: `row` takes `col`, the previous owner of `col` takes its parent column, ...
// until a column without an owner has been taken.  TOP: returns the largest row that changed its column (else 0).
template <int NPL, bool TOP = false>
__device__ __forceinline__ int apply_path(int row, int col, int (&sigma)[NPL], int (&p)[NPL], const int (&parent)[NPL],
                                          int lane, int N) {
    int top = TOP ? row : 0;
    for (int guard = 0; guard <= N; ++guard) {
        int prev_owner = bcast<NPL>(p, col);
        set_at<NPL>(sigma, row, col, lane);
        set_at<NPL>(p, col, row, lane);
        if (prev_owner < 0) break;
        row = prev_owner;
        if (TOP) top = max(top, row);
        col = bcast<NPL>(parent, prev_owner);
    }
    return top;
}

// Inclusive OR-scan over the 64 lanes of a 32-bit value (GFX9 DPP: row shifts, then row broadcasts).
__device__ __forceinline__ unsigned int wave_or_scan32(unsigned int v) {
    v |= (unsigned int)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, false);   // row_shr:1
    v |= (unsigned int)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, false);   // row_shr:2
    v |= (unsigned int)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, false);   // row_shr:4
    v |= (unsigned int)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, false);   // row_shr:8
    v |= (unsigned int)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);   // row_bcast:15 into rows 1, 3
    v |= (unsigned int)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);   // row_bcast:31 into rows 2, 3
    return v;
}
__device__ __forceinline__ unsigned long long wave_or_scan64(unsigned long long v) {
    unsigned int lo = wave_or_scan32((unsigned int)v), hi = wave_or_scan32((unsigned int)(v >> 32));
    return ((unsigned long long)hi << 32) | lo;
}

// Rows >= first_row that have an allowed column below their current one which is not held by an earlier row.
// Only those rows can possibly move to a smaller column; all others are skipped by the lexicographic pass.
template <int NPL, bool SMALL = false>
__device__ __forceinline__ Mask<NPL> rows_with_candidates(const Mask<NPL> (&tm)[NPL], int N, int lane, const int (&sigma)[NPL],
                                                          int first_row) {
    if constexpr (SMALL) {
        const unsigned int own = lane < N ? 1u << (sigma[0] & 31) : 0u;
        const unsigned int taken = wave_or_scan32(own);                  // columns of rows up to and including this one
        Mask<NPL> need = rows_after<NPL, true>(first_row - 1, N);
        need.w[0] &= ballot64(((unsigned int)tm[0].w[0] & (own - 1u) & ~taken) != 0);
        return need;
    }
    // taken[s] = columns held by rows up to and including this lane's row (rows are a permutation: own bit removed below)
    Mask<NPL> taken[NPL], carry;
    carry.clear();
#pragma unroll
    for (int s = 0; s < NPL; ++s) {
        Mask<NPL> own;
        own.clear();
        if (lane + 64 * s < N) own.set(sigma[s]);
#pragma unroll
        for (int k = 0; k < NPL; ++k) {
            taken[s].w[k] = wave_or_scan64(own.w[k]) | carry.w[k];
        }
#pragma unroll
        for (int k = 0; k < NPL; ++k) {
            unsigned int lo = (unsigned int)__builtin_amdgcn_readlane((int)(taken[s].w[k] & 0xFFFFFFFFULL), 63);
            unsigned int hi = (unsigned int)__builtin_amdgcn_readlane((int)(taken[s].w[k] >> 32), 63);
            carry.w[k] = ((unsigned long long)hi << 32) | lo;
        }
    }
    Mask<NPL> need;
#pragma unroll
    for (int s = 0; s < NPL; ++s) {
        const int row = lane + 64 * s;
        bool want = false;
        if (row < N && row >= first_row) {
            Mask<NPL> c = tm[s] & below<NPL>(sigma[s]);
#pragma unroll
            for (int k = 0; k < NPL; ++k) c.w[k] &= ~taken[s].w[k];      // own column is not below itself, so its bit is harmless
            want = c.any();
        }
        need.w[s] = ballot64(want);
    }
    return need;
}

// Turn the perfect matching (sigma: row -> col, p: col -> row) of the graph `tm` into the
// lexicographically smallest perfect matching of that graph, rows < first_row being final already.  Rows are
// settled in ascending order; a row can
// only improve if it has a candidate column (see above), and for such a row one breadth-first search over
// alternating paths through later rows tells which columns can be vacated for it.
// BOUND (the incremental callers, large N): the matching was the lexicographically smallest one of this graph, or of
// one with more edges in rows up to last_row, except that rows up to last_row have changed columns since.  Whether
// row i can move to a smaller column depends only on the edges of rows >= i, on the set of columns these rows hold,
// and on row i's column; for i > last_row none of the three has changed, so such a row still cannot move and is not
// examined.  A re-routing inside this pass raises last_row to the largest row it moved.  (Keeping track of last_row
// costs a 16 x 16 decomposition more than the few searches it saves there; at 64 x 64 it saves a seventh of the time.)
template <int NPL, bool BOUND = false, bool SMALL = false>
__device__ __forceinline__ void lex_smallest(const Mask<NPL> (&tm)[NPL], int N, int lane, int (&sigma)[NPL], int (&p)[NPL],
                                             int first_row, int last_row = 0) {
    const Mask<NPL> all = below<NPL, SMALL>(N);         // every column has an owner here
    for (int round = 0; round <= N; ++round) {
        Mask<NPL> need = rows_with_candidates<NPL, SMALL>(tm, N, lane, sigma, first_row);
        if (BOUND) need = need & below<NPL>(last_row + 1);
        bool changed = false;
        while (need.any() && !changed) {
            const int i = need.first();
            need.reset(i);
            int cur = bcast<NPL>(sigma, i);
            // columns of rows < i are fixed
            Mask<NPL> cand = bcast_mask<NPL>(tm, i) & below<NPL, SMALL>(cur);
#pragma unroll
            for (int s = 0; s < NPL; ++s) cand.w[s] &= ~(ballot64((unsigned int)p[s] < (unsigned int)i) & all.w[s]);
            if (!cand.any()) continue;
            // which columns can be vacated by re-routing rows > i, the column `cur` being free?
            Mask<NPL> reached;
            reached.clear();
            reached.set(cur);
            Mask<NPL> open = rows_after<NPL, SMALL>(i, N);
            int parent[NPL];
#pragma unroll
            for (int s = 0; s < NPL; ++s) parent[s] = -1;
            const int best = cand.first();
            for (int level = 0; level < N; ++level) {
                Mask<NPL> vm = bfs_visit_rows<NPL, SMALL>(tm, reached, lane, open, parent);
                if (!vm.any()) break;
                bfs_reach_cols<NPL, SMALL>(p, vm, all, lane, reached);
                if (reached.test(best)) break;
            }
            Mask<NPL> hit = cand & reached;
            if (hit.any()) {
                set_at<NPL>(p, cur, -1, lane);           // row i gives up its column ...
                const int top = apply_path<NPL, BOUND>(i, hit.first(), sigma, p, parent, lane, N);   // ... and the re-routing ends by taking it
                if (BOUND) last_row = max(last_row, top);
                changed = true;                  // later rows moved: their candidate sets must be recomputed
                first_row = i + 1;
            }
        }
        if (!changed) break;
    }
}

struct Fnv {
    unsigned long long h;
    __device__ __forceinline__ void byte(unsigned int b) { h = (h ^ (unsigned long long)(b & 0xFF)) * FNV_PRIME; }
};

template <int NPL>
__device__ __forceinline__ void emit_matching(const int (&sigma)[NPL], int duration, int N, int lane, int t,
                                              uint8_t* perms_b, int32_t* dur_b, Fnv* fnv) {
    if (perms_b) {
#pragma unroll
        for (int s = 0; s < NPL; ++s) {
            int i = lane + 64 * s;
            if (i < N) perms_b[(size_t)t * N + i] = (uint8_t)sigma[s];
        }
    }
    if (dur_b && lane == 0) dur_b[t] = duration;
    if (fnv) {
        for (int i = 0; i < N; ++i) fnv->byte((unsigned int)bcast<NPL>(sigma, i));
        unsigned int d = (unsigned int)duration;
        for (int k = 0; k < 4; ++k) fnv->byte(d >> (8 * k));
    }
}

// ------------------------------------------------------------------------------ greedy kernel
template <int NPL, typename T, int NW>            // NW: 16-lane rows that hold columns (1, 2 or 4)
__global__ __launch_bounds__(MOE_WAVE)
void greedy_kernel(const int32_t* __restrict__ mats, int N, int kmax, int flags, uint8_t* __restrict__ perms,
                   int32_t* __restrict__ durations, int32_t* __restrict__ counts, int32_t* __restrict__ residual,
                   unsigned long long* __restrict__ hashes, unsigned long long* __restrict__ prof, int prof_cap) {
    extern __shared__ __attribute__((aligned(16))) unsigned char greedy_lds[];
    T* R = reinterpret_cast<T*>(greedy_lds);           // T = uint16_t halves the footprint: twice the wavefronts per CU
    const int lane = threadIdx.x;
    const int b = blockIdx.x;
    // second pass of a batch whose first pass kept the residual in 16 bits: only the matrices that pass marked
    // (an entry did not fit) are decomposed, with the 32-bit residual
    if ((flags & REDO_MARKED) && __builtin_amdgcn_readfirstlane(counts[b]) != NOT_DONE) return;
    const bool profiled = prof != nullptr && b < prof_cap;
    unsigned long long t_cycles = 0, t_real = 0;
    int n_steps = 0, n_searches = 0;
    if (profiled) { t_cycles = __builtin_readcyclecounter(); t_real = wall_clock64(); }
    if (!load_matrix(mats + (size_t)b * N * N, R, N, flags & MOE_DECOMP_ZERO_DIAGONAL, lane)) {
        if (lane == 0) counts[b] = NOT_DONE;            // an entry does not fit 16 bits: left to the second pass
        return;
    }

    // feasible start: u_i = row maximum, v_j = 0  (u_i + v_j >= R_ij)
    int u[NPL], v[NPL], p[NPL], sigma[NPL];
#pragma unroll
    for (int s = 0; s < NPL; ++s) { u[s] = 0; v[s] = 0; p[s] = -1; sigma[s] = -1; }
    int nnz = 0;
    for (int i = 0; i < N; ++i) {
        int m = 0, pos = 0;
#pragma unroll
        for (int s = 0; s < NPL; ++s) {
            int j = lane + 64 * s;
            int x = j < N ? R[i * N + j] : 0;
            m = max(m, x);
            pos += __popcll(ballot64(x > 0));
        }
        m = wave_max(m);
        nnz += pos;
        set_at<NPL>(u, i, m, lane);
    }

    Fnv fnv{FNV_OFFSET};
    uint8_t* perms_b = perms ? perms + (size_t)b * kmax * N : nullptr;
    int32_t* dur_b = durations ? durations + (size_t)b * kmax : nullptr;
    int t = 0;
    while (t < kmax && nnz > 0) {
#pragma unroll
        for (int s = 0; s < NPL; ++s) { p[s] = -1; sigma[s] = -1; }
        // N <= 16: this lane's column of the residual sits in registers for the whole matching (a row picked at run time
        // is then a register selected by a scalar index, not an LDS round trip)
        int Rc[NW == 1 ? 16 : 1];
        if constexpr (NW == 1) {
            const T* col = R + (lane < N ? lane : N - 1);
#pragma unroll
            for (int i = 0; i < 16; ++i) Rc[i] = i < N ? (int)col[i * N] : 0;
        }
        // ---- row reduction: lower u_r until row r has a tight edge, and take that edge if its column is free.
        //      (Duals stay feasible, matched edges are tight; most rows are settled here and skip the search.)
        if constexpr (NPL == 1) {
            // u_r <- max_j (R_rj - v_j) does not depend on the other rows: only the set of taken columns (a scalar
            // mask) links the iterations, so their LDS reads and reductions overlap
            const bool incol = lane < N;
            const T* Rcol = R + (incol ? lane : N - 1);
            unsigned long long taken = 0;
            auto reduce_row = [&](int r, int entry) __attribute__((always_inline)) {
                const int x = incol ? entry - v[0] : INT_MIN;             // lanes without a column never win or tie
                const int m = wave_max_rows<NW>(x);
                const unsigned long long avail = ballot64(x == m) & ~taken;
                // branch-free, so that the reductions of consecutive rows overlap: no free tight column = column -1
                const int pick = __builtin_ffsll((long long)avail) - 1;
                taken |= avail & (0ULL - avail);
                if (lane == pick) p[0] = r;
                if (lane == r) { u[0] = m; sigma[0] = pick; }
            };
            if constexpr (NW == 1) {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (r < N) reduce_row(r, Rc[r]);
            } else {
#pragma unroll 4
                for (int r = 0; r < N; ++r) reduce_row(r, (int)Rcol[r * N]);
            }
        } else {
            Mask<NPL> free_cols = below<NPL>(N);                       // columns nobody has taken yet
            for (int r = 0; r < N; ++r) {
                const T* row = R + r * N;
                int x[NPL], local = INT_MIN;
#pragma unroll
                for (int s = 0; s < NPL; ++s) {
                    const int j = lane + 64 * s;
                    x[s] = j < N ? (int)row[j] - v[s] : INT_MIN;        // lanes without a column never win or tie
                    local = max(local, x[s]);
                }
                const int m = wave_max(local);
                set_at<NPL>(u, r, m, lane);
                int pick = -1;
#pragma unroll
                for (int s = NPL - 1; s >= 0; --s) {
                    const unsigned long long f = ballot64(x[s] == m) & free_cols.w[s];
                    if (f) pick = 64 * s + __builtin_ctzll(f);
                }
                if (pick >= 0) {
                    free_cols.reset(pick);
                    set_at<NPL>(p, pick, r, lane);
                    set_at<NPL>(sigma, r, pick, lane);
                }
            }
        }
        // ---- maximum-weight perfect matching: one shortest augmenting path per row still unmatched
        if constexpr (NPL == 1) {
            // One column per lane: Dijkstra form of the search.  dist_j = length of the shortest alternating path found
            // so far from row r to column j in reduced costs u_i + v_j - R_ij of the duals at the start of the search
            // (they are updated once, at its end); the set of scanned columns is a scalar bit mask.
            const bool incol = lane < N;
            const unsigned long long beyond = N >= 64 ? 0ULL : ~0ULL << N;     // lanes that hold no column count as scanned
            const T* Rcol = R + (incol ? lane : N - 1);
            unsigned long long todo = ballot64(incol && sigma[0] < 0);
            while (todo) {
                const int r = __builtin_ctzll(todo);
                todo &= todo - 1;
                int dist = INT_MAX, way[1] = {-1};
                unsigned long long used = beyond;
                int i0 = r, j0 = -1, D = 0;
                for (int step = 0; step < N; ++step) {
                    const int base = D + rdlane(u[0], i0);               // row i0 entered the tree at distance D
                    const bool open = !__builtin_amdgcn_inverse_ballot_w64(used);
                    int entry;
                    if constexpr (NW == 1) entry = Rc[i0 & 15]; else entry = (int)Rcol[i0 * N];
                    const int cand = open ? base + v[0] - entry : INT_MAX;
                    way[0] = cand < dist ? j0 : way[0];
                    dist = min(dist, cand);
                    const int key = open ? dist : INT_MAX;
                    D = wave_min_rows<NW>(key);                          // (finite: row r is unmatched, so a column is free)
                    const int j1 = __builtin_ctzll(ballot64(key == D));
                    used |= 1ULL << j1;
                    j0 = j1;
                    i0 = rdlane(p[0], j1);
                    ++n_steps;
                    if (i0 < 0) break;
                }
                ++n_searches;
                used &= ~beyond;
                // duals: a scanned column j rises by D - dist_j, its row falls by the same amount, row r falls by D
                // (tree edges stay tight, everything stays feasible, the new path is tight)
                const int sg = sigma[0];
                const int dcol = __shfl(dist, sg < 0 ? 0 : sg);
                const bool rin = sg >= 0 && ((used >> sg) & 1ULL);
                if (__builtin_amdgcn_inverse_ballot_w64(used)) v[0] += D - dist;
                if (lane == r) u[0] -= D; else if (rin) u[0] -= D - dcol;
                // flip the path back to row r
                for (int guard = 0; guard <= N; ++guard) {
                    int j1 = bcast<NPL>(way, j0);
                    int i = r;
                    if (j1 >= 0) i = bcast<NPL>(p, j1);
                    set_at<NPL>(p, j0, i, lane);
                    set_at<NPL>(sigma, i, j0, lane);
                    if (j1 < 0) break;
                    j0 = j1;
                }
            }
        } else {
            // The same search with NPL columns per lane; the sets of scanned columns are NPL uniform masks.
            const Mask<NPL> cols = below<NPL>(N);
            Mask<NPL> todo;
#pragma unroll
            for (int s = 0; s < NPL; ++s) todo.w[s] = ballot64(sigma[s] < 0) & cols.w[s];
            while (todo.any()) {
                const int r = todo.first();
                todo.reset(r);
                int dist[NPL], way[NPL];
                Mask<NPL> used;                                          // columns that do not exist count as scanned
#pragma unroll
                for (int s = 0; s < NPL; ++s) { dist[s] = INT_MAX; way[s] = -1; used.w[s] = ~cols.w[s]; }
                int i0 = r, j0 = -1, D = 0;
                for (int step = 0; step < N; ++step) {
                    const int base = D + bcast<NPL>(u, i0);              // row i0 entered the tree at distance D
                    const T* row = R + i0 * N;
                    int key[NPL], local = INT_MAX;
#pragma unroll
                    for (int s = 0; s < NPL; ++s) {
                        const int j = lane + 64 * s;
                        const bool open = !__builtin_amdgcn_inverse_ballot_w64(used.w[s]);
                        const int entry = (int)row[j < N ? j : N - 1];
                        const int cand = open ? base + v[s] - entry : INT_MAX;
                        way[s] = cand < dist[s] ? j0 : way[s];
                        dist[s] = min(dist[s], cand);
                        key[s] = open ? dist[s] : INT_MAX;
                        local = min(local, key[s]);
                    }
                    D = wave_min(local);                                 // (finite: row r is unmatched, so a column is free)
                    int j1 = -1;
#pragma unroll
                    for (int s = NPL - 1; s >= 0; --s) {
                        const unsigned long long m = ballot64(key[s] == D);
                        if (m) j1 = 64 * s + __builtin_ctzll(m);
                    }
                    used.set(j1);
                    j0 = j1;
                    i0 = bcast<NPL>(p, j1);
                    ++n_steps;
                    if (i0 < 0) break;
                }
                ++n_searches;
                // duals: a scanned column j rises by D - dist_j, its row falls by the same amount, row r falls by D
#pragma unroll
                for (int s = 0; s < NPL; ++s) used.w[s] &= cols.w[s];
                int du[NPL];
#pragma unroll
                for (int s = 0; s < NPL; ++s) {
                    const int sg = sigma[s];                             // the column of this lane's row, if it has one
                    const int src = sg < 0 ? 0 : sg;
                    int dcol = __shfl(dist[0], src & 63);
                    if (NPL > 1) { const int d1 = __shfl(dist[NPL - 1], src & 63); dcol = (src >> 6) ? d1 : dcol; }
                    const bool rin = sg >= 0 && used.test(src);
                    du[s] = lane + 64 * s == r ? D : (rin ? D - dcol : 0);
                }
#pragma unroll
                for (int s = 0; s < NPL; ++s) {
                    if (__builtin_amdgcn_inverse_ballot_w64(used.w[s])) v[s] += D - dist[s];
                    u[s] -= du[s];
                }
                // flip the path back to row r
                for (int guard = 0; guard <= N; ++guard) {
                    int j1 = bcast<NPL>(way, j0);
                    int i = r;
                    if (j1 >= 0) i = bcast<NPL>(p, j1);
                    set_at<NPL>(p, j0, i, lane);
                    set_at<NPL>(sigma, i, j0, lane);
                    if (j1 < 0) break;
                    j0 = j1;
                }
            }
        }
        // ---- canonical optimum: lexicographically smallest perfect matching of the tight graph
        Mask<NPL> tm[NPL];
        {
            int vv[NPL];
#pragma unroll
            for (int s = 0; s < NPL; ++s) vv[s] = v[s];
            if constexpr (NW == 1) {
                tm[0].clear();
                const unsigned long long colmask = below<NPL>(N).w[0];
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (i < N) {
                        const unsigned long long row = ballot64(__builtin_amdgcn_readlane(u[0], i) + vv[0] == Rc[i]) & colmask;
                        if (lane == i) tm[0].w[0] = row;
                    }
            } else {
                build_masks<NPL, T>(R, N, lane, tm, [&](int x, int i, int s) { return bcast<NPL>(u, i) + vv[s] == x; });
            }
        }
        lex_smallest<NPL, false, NPL == 1 && NW <= 2>(tm, N, lane, sigma, p, 0);
        // ---- ship whole entries; the matching lasts as long as its heaviest pair
        int dmax = 0, pos = 0;
#pragma unroll
        for (int s = 0; s < NPL; ++s) {
            int i = lane + 64 * s;
            int x = 0;
            if (i < N) { x = R[i * N + sigma[s]]; R[i * N + sigma[s]] = 0; }
            dmax = max(dmax, x);
            pos += __popcll(ballot64(x > 0));
        }
        dmax = wave_max(dmax);
        nnz -= pos;
        lds_fence();
        emit_matching<NPL>(sigma, dmax, N, lane, t, perms_b, dur_b, hashes ? &fnv : nullptr);
        ++t;
    }
    if (lane == 0) {
        counts[b] = t;
        if (hashes) hashes[b] = fnv.h;
    }
    if (residual) store_matrix(R, residual + (size_t)b * N * N, N, lane);
    if (profiled && lane == 0) {
        prof[4 * (size_t)b + 0] = __builtin_readcyclecounter() - t_cycles;
        prof[4 * (size_t)b + 1] = wall_clock64() - t_real;
        prof[4 * (size_t)b + 2] = (unsigned long long)n_steps;
        prof[4 * (size_t)b + 3] = (unsigned long long)n_searches;
    }
}

// ------------------------------------------------------------------------------ BvN kernel
template <int NPL, bool BOUND>             // BOUND (N > 32): the lexicographic pass stops at the last row the repair moved;
                                           // otherwise (N <= 32) the mask arithmetic is done in 32 bits
__global__ __launch_bounds__(MOE_WAVE)
void bvn_kernel(const int32_t* __restrict__ mats, int N, int kmax, int flags, uint8_t* __restrict__ perms,
                int32_t* __restrict__ durations, int32_t* __restrict__ counts, int32_t* __restrict__ residual,
                int32_t* __restrict__ pad_total, unsigned long long* __restrict__ hashes,
                unsigned long long* __restrict__ prof, int prof_cap) {
    extern __shared__ int32_t R[];
    const int lane = threadIdx.x;
    const int b = blockIdx.x;
    const bool profiled = prof != nullptr && b < prof_cap;
    unsigned long long t_cycles = 0, t_real = 0;
    if (profiled) { t_cycles = __builtin_readcyclecounter(); t_real = wall_clock64(); }
    load_matrix(mats + (size_t)b * N * N, R, N, flags & MOE_DECOMP_ZERO_DIAGONAL, lane);

    // ---- integer padding to equal line sums (north-west-corner fill of the deficits)
    int rdef[NPL], cdef[NPL];
#pragma unroll
    for (int s = 0; s < NPL; ++s) { rdef[s] = 0; cdef[s] = 0; }
    for (int i = 0; i < N; ++i) {
        int part = 0;
#pragma unroll
        for (int s = 0; s < NPL; ++s) {
            int j = lane + 64 * s;
            int x = j < N ? R[i * N + j] : 0;
            cdef[s] += x;                       // column sums accumulate in the column's lane
            part += x;
        }
        set_at<NPL>(rdef, i, wave_sum(part), lane);
    }
    int line_max = 0;
#pragma unroll
    for (int s = 0; s < NPL; ++s) line_max = max(line_max, max(rdef[s], cdef[s]));
    const int target = wave_max(line_max);
#pragma unroll
    for (int s = 0; s < NPL; ++s) {
        int idx = lane + 64 * s;
        rdef[s] = idx < N ? target - rdef[s] : 0;
        cdef[s] = idx < N ? target - cdef[s] : 0;
    }
    {
        int i = 0, j = 0;
        int ri = bcast<NPL>(rdef, 0), cj = bcast<NPL>(cdef, 0);
        for (int guard = 0; guard < 4 * N + 4 && i < N && j < N; ++guard) {   // <= 2N advances + 2N-1 fills
            if (ri == 0) { ++i; if (i < N) ri = bcast<NPL>(rdef, i); continue; }
            if (cj == 0) { ++j; if (j < N) cj = bcast<NPL>(cdef, j); continue; }
            int dl = min(ri, cj);
            if (lane == 0) R[i * N + j] += dl;
            ri -= dl; cj -= dl;
        }
        lds_fence();
    }

    // ---- support masks and number of positive entries
    Mask<NPL> tm[NPL];
    build_masks<NPL, int32_t>(R, N, lane, tm, [](int x, int, int) { return x > 0; });
    int nnz = 0;
#pragma unroll
    for (int s = 0; s < NPL; ++s) {
        int c = 0;
#pragma unroll
        for (int k = 0; k < NPL; ++k) c += __popcll(tm[s].w[k]);
        nnz += wave_sum(c);
    }

    int p[NPL], sigma[NPL];
    const Mask<NPL> all = below<NPL, !BOUND>(N);     // the rows, or the columns, of the matrix
#pragma unroll
    for (int s = 0; s < NPL; ++s) { p[s] = -1; sigma[s] = -1; }
    Fnv fnv{FNV_OFFSET};
    uint8_t* perms_b = perms ? perms + (size_t)b * kmax * N : nullptr;
    int32_t* dur_b = durations ? durations + (size_t)b * kmax : nullptr;
    int t = 0;
    bool broken = false;
    while (t < kmax && nnz > 0 && !broken) {
        // ---- repair, in ascending order of the unmatched rows: row i takes the smallest allowed column that can be
        //      vacated (or is free) by re-routing matched rows > i only.  Rows < i are untouched, so the previous
        //      lexicographically smallest matching stays valid above the first repaired row.
        int first_row = N, last_row = -1;              // range of the rows the repair moves
        bool restricted_ok = true;
        {
            Mask<NPL> unmatched;
#pragma unroll
            for (int s = 0; s < NPL; ++s) unmatched.w[s] = ballot64(sigma[s] < 0) & all.w[s];
            while (unmatched.any() && restricted_ok) {
                const int i = unmatched.first();
                unmatched.reset(i);
                first_row = min(first_row, i);
                Mask<NPL> reached, owned;
#pragma unroll
                for (int s = 0; s < NPL; ++s) {
                    reached.w[s] = ballot64(p[s] < 0) & all.w[s];
                    owned.w[s] = all.w[s] & ~reached.w[s];
                }
                Mask<NPL> open = rows_after<NPL, !BOUND>(i, N);
                int parent[NPL];
#pragma unroll
                for (int s = 0; s < NPL; ++s) parent[s] = -1;
                const Mask<NPL> allowed = bcast_mask<NPL>(tm, i);
                const int best = allowed.any() ? allowed.first() : -1;
                for (int level = 0; level <= N; ++level) {
                    if (best >= 0 && reached.test(best)) break;
                    Mask<NPL> vm = bfs_visit_rows<NPL, !BOUND>(tm, reached, lane, open, parent);
                    if (!vm.any()) break;
                    bfs_reach_cols<NPL, !BOUND>(p, vm, owned, lane, reached);
                }
                Mask<NPL> hit = allowed & reached;
                if (hit.any()) {
                    const int top = apply_path<NPL, BOUND>(i, hit.first(), sigma, p, parent, lane, N);
                    if (BOUND) last_row = max(last_row, top);
                } else {
                    restricted_ok = false;
                }
            }
        }
        if (!restricted_ok) {
            // general repair: every free column looks for an unmatched row along an alternating path through any rows
            first_row = 0;
            last_row = N - 1;
            Mask<NPL> free_cols;
#pragma unroll
            for (int s = 0; s < NPL; ++s) free_cols.w[s] = ballot64(p[s] < 0) & all.w[s];
            while (free_cols.any() && !broken) {
                const int cf = free_cols.first();
                free_cols.reset(cf);
                Mask<NPL> reached;
                reached.clear();
                reached.set(cf);
                Mask<NPL> open = all, owned;
#pragma unroll
                for (int s = 0; s < NPL; ++s) owned.w[s] = all.w[s] & ~ballot64(p[s] < 0);
                int parent[NPL];
#pragma unroll
                for (int s = 0; s < NPL; ++s) parent[s] = -1;
                int target_row = -1;
                for (int level = 0; level <= N; ++level) {
                    Mask<NPL> vm = bfs_visit_rows<NPL>(tm, reached, lane, open, parent);
                    if (!vm.any()) break;
                    Mask<NPL> um;                    // newly visited rows that are unmatched
#pragma unroll
                    for (int s = 0; s < NPL; ++s) um.w[s] = vm.w[s] & ballot64(sigma[s] < 0);
                    if (um.any()) { target_row = um.first(); break; }
                    bfs_reach_cols<NPL>(p, vm, owned, lane, reached);
                }
                if (target_row < 0) { broken = true; break; }     // impossible for equal line sums
                apply_path<NPL>(target_row, bcast<NPL>(parent, target_row), sigma, p, parent, lane, N);
            }
        }
        if (broken) break;
        lex_smallest<NPL, BOUND, !BOUND>(tm, N, lane, sigma, p, first_row < N ? (restricted_ok ? first_row + 1 : 0) : N, last_row);
        // ---- coefficient = smallest entry on the matching; subtract it
        int x[NPL], lmin = INT_MAX;
#pragma unroll
        for (int s = 0; s < NPL; ++s) {
            int i = lane + 64 * s;
            x[s] = i < N ? R[i * N + sigma[s]] : INT_MAX;
            lmin = min(lmin, x[s]);
        }
        const int lambda = BOUND ? wave_min(lmin) : wave_min_rows<2>(lmin);      // (N <= 32: two 16-lane rows)
        emit_matching<NPL>(sigma, lambda, N, lane, t, perms_b, dur_b, hashes ? &fnv : nullptr);
        ++t;
        // entries equal to the coefficient die (lanes without a row hold INT_MAX, which no coefficient reaches)
        Mask<NPL> dead_rows;
#pragma unroll
        for (int s = 0; s < NPL; ++s) {
            const int i = lane + 64 * s;
            const bool dead = x[s] == lambda;
            dead_rows.w[s] = ballot64(dead);
            if (i < N) R[i * N + sigma[s]] = x[s] - lambda;
            if (dead) {
                if constexpr (!BOUND) tm[s].w[0] = (unsigned int)tm[s].w[0] & ~(1u << (sigma[s] & 31));
                else tm[s].reset(sigma[s]);
                sigma[s] = -1;
            }
        }
#pragma unroll
        for (int s = 0; s < NPL; ++s) {
            nnz -= __popcll(dead_rows.w[s]);
            // (a column without an owner tests some bit and, if that is set, becomes ownerless once more)
            bool lost;
            if constexpr (!BOUND) lost = (((unsigned int)dead_rows.w[0] >> (p[s] & 31)) & 1u) != 0;
            else lost = dead_rows.test(p[s] & (64 * NPL - 1));
            if (lost) p[s] = -1;
        }
        lds_fence();
    }
    if (lane == 0) {
        counts[b] = broken ? -1 : t;
        if (pad_total) pad_total[b] = target;
        if (hashes) hashes[b] = fnv.h;
    }
    if (residual) store_matrix(R, residual + (size_t)b * N * N, N, lane);
    if (profiled && lane == 0) {
        prof[4 * (size_t)b + 0] = __builtin_readcyclecounter() - t_cycles;
        prof[4 * (size_t)b + 1] = wall_clock64() - t_real;
        prof[4 * (size_t)b + 2] = 0;
        prof[4 * (size_t)b + 3] = 0;
    }
}

// ------------------------------------------------------------------------------ Sinkhorn-Knopp + floating-point BvN kernel
// Section 3.1: the matrix is first scaled towards unit line sums, then decomposed.  Double precision; the scaled
// matrix (N x N doubles, up to 128 KiB) lives in LDS.  Every sum runs in index order inside one lane (lane i owns
// row i in the row sweep, lane j owns column j in the column sweep), every division is a plain IEEE division: the
// result does not depend on how lanes are scheduled and can be reproduced bit for bit by a sequential program.
__device__ __forceinline__ double wave_min_f64(double x) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x = fmin(x, __shfl_xor(x, off));
    return x;
}
__device__ __forceinline__ double wave_max_f64(double x) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x = fmax(x, __shfl_xor(x, off));
    return x;
}

template <int NPL, bool BOUND>
__global__ __launch_bounds__(MOE_WAVE)
void sinkhorn_bvn_kernel(const int32_t* __restrict__ mats, int N, int kmax, int flags, int iters, double eps,
                         uint8_t* __restrict__ perms, double* __restrict__ coeffs, int32_t* __restrict__ counts,
                         double* __restrict__ scaled, double* __restrict__ residual, double* __restrict__ deviation) {
    extern __shared__ double X[];
    const int lane = threadIdx.x;
    const int b = blockIdx.x;
    {
        const int32_t* A = mats + (size_t)b * N * N;
        const bool zd = flags & MOE_DECOMP_ZERO_DIAGONAL;
        for (int x = lane; x < N * N; x += MOE_WAVE) X[x] = (zd && x / N == x % N) ? 0.0 : (double)A[x];
        lds_fence();
    }
    // ---- Sinkhorn-Knopp sweeps: rows, then columns; a line whose sum is zero is left alone
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < NPL; ++s) {
            const int i = lane + 64 * s;
            if (i < N) {
                double sum = 0.0;
                for (int j = 0; j < N; ++j) sum += X[i * N + j];
                if (sum > 0.0)
                    for (int j = 0; j < N; ++j) X[i * N + j] = X[i * N + j] / sum;
            }
        }
        lds_fence();
#pragma unroll
        for (int s = 0; s < NPL; ++s) {
            const int j = lane + 64 * s;
            if (j < N) {
                double sum = 0.0;
                for (int i = 0; i < N; ++i) sum += X[i * N + j];
                if (sum > 0.0)
                    for (int i = 0; i < N; ++i) X[i * N + j] = X[i * N + j] / sum;
            }
        }
        lds_fence();
    }
    {
        double dev = 0.0;
#pragma unroll
        for (int s = 0; s < NPL; ++s) {
            const int i = lane + 64 * s;
            if (i < N) {
                double sum = 0.0;
                for (int j = 0; j < N; ++j) sum += X[i * N + j];
                dev = fmax(dev, sum > 1.0 ? sum - 1.0 : 1.0 - sum);
            }
        }
        dev = wave_max_f64(dev);
        if (deviation && lane == 0) deviation[b] = dev;
    }
    if (scaled) {
        double* out = scaled + (size_t)b * N * N;
        for (int x = lane; x < N * N; x += MOE_WAVE) out[x] = X[x];
    }

    // ---- BvN on the scaled matrix: perfect matchings inside {X > eps}, repaired incrementally (as bvn_kernel)
    Mask<NPL> tm[NPL];
    build_masks<NPL, double>(X, N, lane, tm, [eps](double x, int, int) { return x > eps; });
    int nnz = 0;
#pragma unroll
    for (int s = 0; s < NPL; ++s) {
        int c = 0;
#pragma unroll
        for (int k = 0; k < NPL; ++k) c += __popcll(tm[s].w[k]);
        nnz += wave_sum(c);
    }
    int p[NPL], sigma[NPL];
    const Mask<NPL> all = below<NPL, !BOUND>(N);     // the rows, or the columns, of the matrix
#pragma unroll
    for (int s = 0; s < NPL; ++s) { p[s] = -1; sigma[s] = -1; }
    uint8_t* perms_b = perms ? perms + (size_t)b * kmax * N : nullptr;
    double* coef_b = coeffs ? coeffs + (size_t)b * kmax : nullptr;
    int t = 0;
    bool stuck = false;
    while (t < kmax && nnz > 0 && !stuck) {
        int first_row = N, last_row = -1;              // range of the rows the repair moves
        bool restricted_ok = true;
        {
            Mask<NPL> unmatched;
#pragma unroll
            for (int s = 0; s < NPL; ++s) unmatched.w[s] = ballot64(sigma[s] < 0) & all.w[s];
            while (unmatched.any() && restricted_ok) {
                const int i = unmatched.first();
                unmatched.reset(i);
                first_row = min(first_row, i);
                Mask<NPL> reached, owned;
#pragma unroll
                for (int s = 0; s < NPL; ++s) {
                    reached.w[s] = ballot64(p[s] < 0) & all.w[s];
                    owned.w[s] = all.w[s] & ~reached.w[s];
                }
                Mask<NPL> open = rows_after<NPL, !BOUND>(i, N);
                int parent[NPL];
#pragma unroll
                for (int s = 0; s < NPL; ++s) parent[s] = -1;
                const Mask<NPL> allowed = bcast_mask<NPL>(tm, i);
                const int best = allowed.any() ? allowed.first() : -1;
                for (int level = 0; level <= N; ++level) {
                    if (best >= 0 && reached.test(best)) break;
                    Mask<NPL> vm = bfs_visit_rows<NPL, !BOUND>(tm, reached, lane, open, parent);
                    if (!vm.any()) break;
                    bfs_reach_cols<NPL, !BOUND>(p, vm, owned, lane, reached);
                }
                Mask<NPL> hit = allowed & reached;
                if (hit.any()) {
                    const int top = apply_path<NPL, BOUND>(i, hit.first(), sigma, p, parent, lane, N);
                    if (BOUND) last_row = max(last_row, top);
                } else {
                    restricted_ok = false;
                }
            }
        }
        if (!restricted_ok) {
            first_row = 0;
            last_row = N - 1;
            Mask<NPL> free_cols;
#pragma unroll
            for (int s = 0; s < NPL; ++s) free_cols.w[s] = ballot64(p[s] < 0) & all.w[s];
            while (free_cols.any() && !stuck) {
                const int cf = free_cols.first();
                free_cols.reset(cf);
                Mask<NPL> reached;
                reached.clear();
                reached.set(cf);
                Mask<NPL> open = all, owned;
#pragma unroll
                for (int s = 0; s < NPL; ++s) owned.w[s] = all.w[s] & ~ballot64(p[s] < 0);
                int parent[NPL];
#pragma unroll
                for (int s = 0; s < NPL; ++s) parent[s] = -1;
                int target_row = -1;
                for (int level = 0; level <= N; ++level) {
                    Mask<NPL> vm = bfs_visit_rows<NPL>(tm, reached, lane, open, parent);
                    if (!vm.any()) break;
                    Mask<NPL> um;
#pragma unroll
                    for (int s = 0; s < NPL; ++s) um.w[s] = vm.w[s] & ballot64(sigma[s] < 0);
                    if (um.any()) { target_row = um.first(); break; }
                    bfs_reach_cols<NPL>(p, vm, owned, lane, reached);
                }
                if (target_row < 0) { stuck = true; break; }      // the support holds no perfect matching: the scaling was approximate
                apply_path<NPL>(target_row, bcast<NPL>(parent, target_row), sigma, p, parent, lane, N);
            }
        }
        if (stuck) break;
        lex_smallest<NPL, BOUND, !BOUND>(tm, N, lane, sigma, p, first_row < N ? (restricted_ok ? first_row + 1 : 0) : N, last_row);
        double x[NPL], lmin = 1.0e300;
#pragma unroll
        for (int s = 0; s < NPL; ++s) {
            const int i = lane + 64 * s;
            x[s] = i < N ? X[i * N + sigma[s]] : 1.0e300;
            lmin = fmin(lmin, x[s]);
        }
        const double lambda = wave_min_f64(lmin);
        if (perms_b) {
#pragma unroll
            for (int s = 0; s < NPL; ++s) {
                const int i = lane + 64 * s;
                if (i < N) perms_b[(size_t)t * N + i] = (uint8_t)sigma[s];
            }
        }
        if (coef_b && lane == 0) coef_b[t] = lambda;
        ++t;
        Mask<NPL> dead_rows;
#pragma unroll
        for (int s = 0; s < NPL; ++s) {
            const int i = lane + 64 * s;
            bool dead = false;
            if (i < N) {
                const double nx = x[s] - lambda;
                X[i * N + sigma[s]] = nx;
                dead = !(nx > eps);
            }
            if (dead) { tm[s].reset(sigma[s]); sigma[s] = -1; }
            dead_rows.w[s] = ballot64(dead);
        }
#pragma unroll
        for (int s = 0; s < NPL; ++s) {
            nnz -= __popcll(dead_rows.w[s]);
            if (p[s] >= 0 && dead_rows.test(p[s])) p[s] = -1;
        }
        lds_fence();
    }
    if (lane == 0) counts[b] = t;
    if (residual) {
        double* out = residual + (size_t)b * N * N;
        for (int x = lane; x < N * N; x += MOE_WAVE) out[x] = X[x];
    }
}

std::atomic<unsigned long long*> g_prof{nullptr};     // moe_decompose_profile: per-matrix counters of the following calls
std::atomic<int> g_prof_cap{0};

std::atomic<int> g_cus[64];
int compute_units() {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
    n = g_cus[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        g_cus[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

moe_status check_args(const int32_t* mats, int B, int N, int kmax, int32_t* counts) {
    if (B < 0 || N < 1 || kmax < 0 || !counts) return MOE_ERR_INVALID_ARG;
    if (B > 0 && !mats) return MOE_ERR_INVALID_ARG;
    if (N > MOE_MAX_RANKS) return MOE_ERR_UNSUPPORTED_SHAPE;
    return MOE_OK;
}

}  // namespace

extern "C" moe_status moe_decompose_profile(uint64_t* counters, int capacity) {
    if (capacity < 0 || (capacity > 0 && !counters)) return MOE_ERR_INVALID_ARG;
    g_prof.store(capacity > 0 ? (unsigned long long*)counters : nullptr, std::memory_order_relaxed);
    g_prof_cap.store(capacity, std::memory_order_relaxed);
    return MOE_OK;
}

extern "C" moe_status moe_decompose_greedy(const int32_t* mats, int B, int N, int kmax, int flags, uint8_t* perms,
                                           int32_t* durations, int32_t* counts, int32_t* residual, uint64_t* hashes,
                                           void* hip_stream) {
    moe_status st = check_args(mats, B, N, kmax, counts);
    if (st != MOE_OK) return st;
    if ((flags & MOE_DECOMP_RESIDUAL_I32) && (flags & MOE_DECOMP_RESIDUAL_U16)) return MOE_ERR_INVALID_ARG;
    if (B == 0) return MOE_OK;
    hipStream_t s = (hipStream_t)hip_stream;
    // Residual in 16 bits where the entries allow it: half the LDS per matrix, so more wavefronts share a compute unit.
    // That pays when LDS, not the number of matrices, limits how many are in flight: matrices of more than 64 ranks
    // (64 KiB each in 32 bits: two per compute unit) in batches that fill the chip more than twice over.  A matrix
    // with an entry of 65536 or more is marked by the 16-bit pass and decomposed by a second launch with the 32-bit
    // residual, in which all other workgroups exit at once.
    bool narrow = N > 64 && B > 2 * compute_units();
    if (flags & MOE_DECOMP_RESIDUAL_I32) narrow = false;
    if (flags & MOE_DECOMP_RESIDUAL_U16) narrow = true;
    const int kflags = flags & MOE_DECOMP_ZERO_DIAGONAL;
    unsigned long long* prof = g_prof.load(std::memory_order_relaxed);
    const int prof_cap = g_prof_cap.load(std::memory_order_relaxed);
    const size_t lds32 = (size_t)N * N * sizeof(int32_t);
    auto wide = N <= 16 ? greedy_kernel<1, int32_t, 1> : N <= 32 ? greedy_kernel<1, int32_t, 2>
              : N <= 64 ? greedy_kernel<1, int32_t, 4> : greedy_kernel<2, int32_t, 4>;
    if (narrow) {
        auto kern = N <= 16 ? greedy_kernel<1, uint16_t, 1> : N <= 32 ? greedy_kernel<1, uint16_t, 2>
                  : N <= 64 ? greedy_kernel<1, uint16_t, 4> : greedy_kernel<2, uint16_t, 4>;
        moe::LaunchScope k("greedy_kernel", s);
        hipLaunchKernelGGL(kern, dim3(B), dim3(MOE_WAVE), lds32 / 2, s, mats, N, kmax, kflags, perms, durations, counts, residual,
                           (unsigned long long*)hashes, prof, prof_cap);
        st = k.done();
        if (st != MOE_OK) return st;
        moe::LaunchScope k2("greedy_redo_kernel", s);
        hipLaunchKernelGGL(wide, dim3(B), dim3(MOE_WAVE), lds32, s, mats, N, kmax, kflags | REDO_MARKED, perms, durations, counts,
                           residual, (unsigned long long*)hashes, prof, prof_cap);
        return k2.done();
    }
    moe::LaunchScope k("greedy_kernel", s);
    hipLaunchKernelGGL(wide, dim3(B), dim3(MOE_WAVE), lds32, s, mats, N, kmax, kflags, perms, durations, counts, residual,
                       (unsigned long long*)hashes, prof, prof_cap);
    return k.done();
}

extern "C" moe_status moe_decompose_bvn(const int32_t* mats, int B, int N, int kmax, int flags, uint8_t* perms,
                                        int32_t* durations, int32_t* counts, int32_t* residual, int32_t* pad_total,
                                        uint64_t* hashes, void* hip_stream) {
    moe_status st = check_args(mats, B, N, kmax, counts);
    if (st != MOE_OK) return st;
    if (B == 0) return MOE_OK;
    hipStream_t s = (hipStream_t)hip_stream;
    const size_t lds = (size_t)N * N * sizeof(int32_t);
    moe::LaunchScope k("bvn_kernel", s);
    auto kern = N <= 32 ? bvn_kernel<1, false> : (N <= 64 ? bvn_kernel<1, true> : bvn_kernel<2, true>);
    hipLaunchKernelGGL(kern, dim3(B), dim3(MOE_WAVE), lds, s, mats, N, kmax, flags, perms, durations, counts, residual, pad_total,
                       (unsigned long long*)hashes, g_prof.load(std::memory_order_relaxed), g_prof_cap.load(std::memory_order_relaxed));
    return k.done();
}

extern "C" moe_status moe_decompose_sinkhorn_bvn(const int32_t* mats, int B, int N, int kmax, int flags, int sweeps, double eps,
                                                 uint8_t* perms, double* coeffs, int32_t* counts, double* scaled,
                                                 double* residual, double* deviation, void* hip_stream) {
    moe_status st = check_args(mats, B, N, kmax, counts);
    if (st != MOE_OK) return st;
    if (sweeps < 0 || !(eps >= 0.0)) return MOE_ERR_INVALID_ARG;
    if (B == 0) return MOE_OK;
    hipStream_t s = (hipStream_t)hip_stream;
    const size_t lds = (size_t)N * N * sizeof(double);
    static moe::DeviceOnce attr;
    int dev;
    if (attr.needed(dev)) {
        hipError_t e = hipFuncSetAttribute((const void*)sinkhorn_bvn_kernel<2, true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           MOE_MAX_RANKS * MOE_MAX_RANKS * (int)sizeof(double));
        if (e != hipSuccess) { moe::note_hip_error(e, "hipFuncSetAttribute(MaxDynamicSharedMemorySize)"); return MOE_ERR_HIP; }
        attr.mark(dev);
    }
    moe::LaunchScope k("sinkhorn_bvn_kernel", s);
    auto kern = N <= 32 ? sinkhorn_bvn_kernel<1, false> : (N <= 64 ? sinkhorn_bvn_kernel<1, true> : sinkhorn_bvn_kernel<2, true>);
    hipLaunchKernelGGL(kern, dim3(B), dim3(MOE_WAVE), lds, s, mats, N, kmax, flags, sweeps, eps, perms, coeffs, counts, scaled,
                       residual, deviation);
    return k.done();
}

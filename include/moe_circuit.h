/*
 * moe_circuit.h -- C ABI of the MI355X (gfx950) library for one receiving GPU's MoE
 * dispatch -> compute -> combine under a circuit schedule.
 *
 * Paper: "Birkhoff Decompositions and Photonic Interconnects - Wait! Don't Forget the Compute!"
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers unless a comment says "host".  The caller owns every
 *     buffer; the library neither allocates nor frees device memory.  State kept between calls:
 *     the optional kernel-timing table, the settings of the test / measurement hooks
 *     (moe_ffn_tile_override, moe_decompose_profile), per-device facts looked up once (number of
 *     compute units, kernel attributes) and the fixed work area of moe_slice_table_static.
 *   - `hip_stream` is a hipStream_t (NULL = the default stream).  Calls validate their arguments
 *     on the host, enqueue their kernels on that stream and return without synchronising.
 *   - Return value: MOE_OK or a negative moe_status.  Nothing throws across this boundary.  On an
 *     argument error nothing has been enqueued.
 *   - Results are deterministic: the same input bytes give the same output bytes.
 *   - Notation: N ranks, E experts (E % N == 0, expert e lives on rank e / (E/N), E_loc = E/N),
 *     T tokens per rank, topk experts per token, r the receiving rank, kmax the cap on matchings.
 */
#ifndef MOE_CIRCUIT_H
#define MOE_CIRCUIT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int moe_status;
#define MOE_OK                     0
#define MOE_ERR_INVALID_ARG       (-1)  /* NULL where a buffer is required, negative size, ... */
#define MOE_ERR_UNSUPPORTED_SHAPE (-2)  /* shape outside what the kernels are built for       */
#define MOE_ERR_WORKSPACE         (-3)  /* workspace missing or too small                      */
#define MOE_ERR_HIP               (-4)  /* a HIP runtime call failed (see moe_last_hip_error)  */

#define MOE_MAX_RANKS   128     /* largest N of the decomposition kernels (residual lives in LDS) */
#define MOE_MAX_EXPERTS 4096    /* largest E of the histogram kernel                              */

/* flags of the decomposition calls */
#define MOE_DECOMP_ZERO_DIAGONAL 1  /* treat the diagonal (tokens whose expert is local) as zero */
/* moe_decompose_greedy keeps the residual of a matrix on chip, in 16 bits when that lets more matrices share a
 * compute unit (N > 64 in batches that fill the chip more than twice over); a matrix with an entry >= 65536 is
 * then decomposed again with a 32-bit residual by a second launch.  Results do not depend on the choice.  The two
 * flags below pin it (tests, measurements); giving both is an error. */
#define MOE_DECOMP_RESIDUAL_I32  2  /* 32-bit residual for every matrix                                        */
#define MOE_DECOMP_RESIDUAL_U16  4  /* 16-bit first, whatever N and the batch size                             */

/* weight formats of moe_expert_ffn_sliced */
#define MOE_W_BF16            0   /* bfloat16                                                     */
#define MOE_W_FP8_E4M3_B128   1   /* OCP FP8 E4M3 codes (S.1111.111 = NaN, no infinities) + one float
                                     scale per 128 x 128 block                                   */

/* ---------------------------------------------------------------------------------------------
 * moe_route_histogram -- Section 2.1 (dispatch) / Section 3 (the all-to-all communication
 * matrix between ranks).  For each of L independent layers:
 *     expert_counts[l][s][e] = #{(t, j) : ids[l][s][t][j] == e}
 *     traffic[l][s][q]       = sum of expert_counts[l][s][e] over the experts e of rank q
 * i.e. every (token, expert) assignment is counted once, local ones (q == s) included.
 *   ids            in   int32 [L][N][T][topk]; values outside [0, E) are ignored
 *   traffic        out  int32 [L][N][N], row = source rank, column = destination rank; overwritten
 *   expert_counts  out  int32 [L][N][E], overwritten; may be NULL
 * Limits: 1 <= N, E % N == 0, E <= MOE_MAX_EXPERTS, L*N*T*topk < 2^31.
 * ------------------------------------------------------------------------------------------- */
moe_status moe_route_histogram(const int32_t* ids, int L, int N, int T, int topk, int E,
                               int32_t* traffic, int32_t* expert_counts, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * moe_decompose_greedy -- Section 3.2 (greedy max-weight decomposition).  For each of B
 * matrices: R <- A; while R != 0 and fewer than kmax matchings were emitted: sigma <- a
 * maximum-weight perfect matching of R (among equally heavy ones the lexicographically
 * smallest sequence sigma(0), sigma(1), ...); duration <- max_i R[i][sigma(i)] (a matching lasts
 * as long as its heaviest pair, Section 3.3); R[i][sigma(i)] <- 0 for all i (each matched pair
 * ships everything it has).
 *   mats       in   int32 [B][N][N], entries >= 0, N * max entry < 2^31
 *   perms      out  uint8 [B][kmax][N], perms[b][t][i] = sigma_t(i); may be NULL
 *   durations  out  int32 [B][kmax]; may be NULL
 *   counts     out  int32 [B]  number of matchings emitted (<= kmax)
 *   residual   out  int32 [B][N][N]  R at exit (all zero unless the cap stopped it); may be NULL
 *   hashes     out  uint64 [B]; may be NULL.  FNV-1a (64 bit) over the byte stream
 *                   sigma_t(0..N-1), duration_t (4 bytes little endian), t = 0..count-1
 * Entries of perms / durations at t >= counts[b] are left untouched.
 * Limits: 1 <= N <= MOE_MAX_RANKS, kmax >= 0, B >= 0.
 * ------------------------------------------------------------------------------------------- */
moe_status moe_decompose_greedy(const int32_t* mats, int B, int N, int kmax, int flags,
                                uint8_t* perms, int32_t* durations, int32_t* counts,
                                int32_t* residual, uint64_t* hashes, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * moe_decompose_bvn -- Section 3.1 (Birkhoff-von Neumann decomposition, the baseline).  BvN
 * needs equal line sums; instead of the paper's Sinkhorn-Knopp scaling the matrix is balanced
 * exactly with integer padding: Tstar = the largest row or column sum, the row and column
 * deficits are filled by the north-west-corner rule, P = A + padding.  Then, while P != 0 and
 * fewer than kmax matchings: sigma <- the lexicographically smallest perfect matching inside
 * {P > 0}; lambda <- min_i P[i][sigma(i)]; P -= lambda * P_sigma.  Uncapped, sum(lambda) = Tstar
 * and sum(lambda_t * P_sigma_t) = A + padding exactly; at most (N-1)^2 + 1 matchings.
 *   arguments as moe_decompose_greedy; durations holds lambda_t; residual is the padded residual;
 *   pad_total  out  int32 [B]  Tstar; may be NULL
 * ------------------------------------------------------------------------------------------- */
moe_status moe_decompose_bvn(const int32_t* mats, int B, int N, int kmax, int flags,
                             uint8_t* perms, int32_t* durations, int32_t* counts,
                             int32_t* residual, int32_t* pad_total, uint64_t* hashes,
                             void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * moe_decompose_profile -- measurement hook, not meant for production callers.  While a buffer is
 * set, moe_decompose_greedy and moe_decompose_bvn record, for every matrix b < capacity, four
 * 64-bit counters at counters[4 * b]: [0] shader clock cycles and [1] ticks of the constant
 * 100 MHz real-time counter between the wavefront's first and last instruction (their ratio is the
 * shader clock the kernel ran at), [2] steps of the augmenting-path searches (one step scans one
 * row of the residual and settles one column) and [3] number of such searches (greedy only; zero
 * for BvN).  The decompositions themselves are unchanged.
 *   counters  device uint64 [4 * capacity], or NULL with capacity 0 to switch recording off
 * Process-wide; the buffer must stay valid until the calls that were enqueued while it was set
 * have finished.
 * ------------------------------------------------------------------------------------------- */
moe_status moe_decompose_profile(uint64_t* counters, int capacity);

/* ---------------------------------------------------------------------------------------------
 * moe_decompose_sinkhorn_bvn -- Section 3.1 as the paper describes it: Sinkhorn-Knopp scaling
 * towards a doubly stochastic matrix, then Birkhoff-von Neumann on the scaled matrix.  Double
 * precision.  X <- A (diagonal zeroed with MOE_DECOMP_ZERO_DIAGONAL); `sweeps` times: every row
 * with a positive sum is divided by its sum, then every column (sums taken in index order).  Then,
 * while fewer than kmax matchings were emitted and {X > eps} holds a perfect matching: sigma <- the
 * lexicographically smallest one; coefficient <- min_i X[i][sigma(i)]; X[i][sigma(i)] -= it.
 * The paper gives neither a number of sweeps nor a tolerance; both are arguments.  The scaling is
 * approximate (and cannot converge at all on a matrix without total support), so the loop may stop
 * with crumbs left: they are returned in `residual`.
 *   mats       in   int32 [B][N][N], entries >= 0
 *   perms      out  uint8 [B][kmax][N]; may be NULL
 *   coeffs     out  double [B][kmax]  the convex weights lambda_t; may be NULL
 *   counts     out  int32 [B]
 *   scaled     out  double [B][N][N]  X after the sweeps; may be NULL
 *   residual   out  double [B][N][N]  X at exit; may be NULL
 *   deviation  out  double [B]  max_i |row sum of the scaled matrix - 1|; may be NULL
 * Limits as moe_decompose_greedy; sweeps >= 0, eps >= 0.  Results are bit-reproducible: every sum is
 * taken in index order by one lane.
 * ------------------------------------------------------------------------------------------- */
moe_status moe_decompose_sinkhorn_bvn(const int32_t* mats, int B, int N, int kmax, int flags, int sweeps, double eps,
                                      uint8_t* perms, double* coeffs, int32_t* counts, double* scaled,
                                      double* residual, double* deviation, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * moe_slice_table -- Sections 2.2 and 4.1: per matching a receiver hears from exactly one
 * source and its experts may start as soon as that batch has arrived.  For receiving rank r
 * this builds the row boundaries of the token batch each matching delivers.
 * Slices: 0 = local assignments (source r); 1 + t = delivered by matching t, t < kmax (empty for
 * t >= *count); kmax + 1 = everything the capped schedule did not ship.  On matching t the pair
 * (s, sigma_t(s) == r) ships min(remaining, duration_t) assignments, first-in-first-out in the
 * order (token, slot) of source s restricted to experts on r.  Inside a slice rows are grouped
 * by local expert.
 *   ids        in   int32 [N][T][topk]
 *   traffic    in   int32 [N][N]   (from moe_route_histogram, diagonal included)
 *   perms      in   uint8 [kmax][N], durations in int32 [kmax], count in int32 [1]
 *   offsets    out  int32 [(kmax+2)*E_loc + 1], group g = slice*E_loc + local expert,
 *                   offsets[0] = 0, offsets[last] = rows received by r
 *   workspace       moe_slice_table_workspace_bytes(N, kmax, E) bytes
 * ------------------------------------------------------------------------------------------- */
size_t     moe_slice_table_workspace_bytes(int N, int kmax, int E);
moe_status moe_slice_table(const int32_t* ids, int N, int T, int topk, int E, int r,
                           const int32_t* traffic, const uint8_t* perms, const int32_t* durations,
                           const int32_t* count, int kmax, int32_t* offsets,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * moe_slice_table_static -- moe_slice_table for callers that cannot hand over a workspace they
 * allocated: code under HIP graph capture, tight serving loops, harnesses that forbid device
 * allocation.  The work area is a fixed array of MOE_SLICE_TABLE_STATIC_BYTES inside the library's
 * device image (every GPU the library runs on holds one for the life of the process); the call
 * allocates and frees nothing.  Same arguments, same kernels and same results as moe_slice_table.
 * Returns MOE_ERR_WORKSPACE when moe_slice_table_workspace_bytes(N, kmax, E) exceeds
 * MOE_SLICE_TABLE_STATIC_BYTES (nothing is enqueued then): use moe_slice_table for such schedules.
 * All calls on one GPU share that GPU's work area: two calls that overlap in time on the same GPU
 * (different streams, or different threads) race; calls on one stream are ordered and safe.
 * ------------------------------------------------------------------------------------------- */
#define MOE_SLICE_TABLE_STATIC_BYTES (4u << 20)
moe_status moe_slice_table_static(const int32_t* ids, int N, int T, int topk, int E, int r,
                                  const int32_t* traffic, const uint8_t* perms, const int32_t* durations,
                                  const int32_t* count, int kmax, int32_t* offsets, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * moe_slice_table_rows -- moe_slice_table plus the row map that turns "dispatch" into a gather
 * (Section 2.1: dispatch sends each token to its experts, combine returns the results): rows
 * reach rank r source by source, each source in its (token, slot) order; the schedule wants them
 * slice by slice.  For every schedule row m in [0, offsets[last]) (slice-major, then local
 * expert, then source rank, then arrival order):
 *   row_arrival[m]     = position of that assignment in the arrival order (0 .. M-1)
 *   row_assignment[m]  = s * T * topk + t * topk + slot, its index in ids
 * Either output may be NULL (not both).  Other arguments as moe_slice_table; workspace of
 * moe_slice_table_rows_workspace_bytes(N, kmax, E) bytes.
 * Limits: as moe_slice_table, and (kmax + 1) * E_loc <= 8192, E_loc <= 64.
 * ------------------------------------------------------------------------------------------- */
size_t     moe_slice_table_rows_workspace_bytes(int N, int kmax, int E);
moe_status moe_slice_table_rows(const int32_t* ids, int N, int T, int topk, int E, int r,
                                const int32_t* traffic, const uint8_t* perms, const int32_t* durations,
                                const int32_t* count, int kmax, int32_t* offsets,
                                int32_t* row_arrival, int32_t* row_assignment,
                                void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * moe_expert_ffn_sliced -- Section 2.1 (the compute step between dispatch and combine), issued
 * for all slices of a schedule at once so that no launch is paid per matching (Section 2.2: what
 * a small batch costs is mostly fixed overhead).
 * For every group g = slice*E_loc + e and every row m in [offsets[g], offsets[g+1]):
 *     y[m] = ( silu(x[m] Wg_e^T) * (x[m] Wu_e^T) ) Wd_e^T ,  silu(z) = z / (1 + exp(-z))
 * with bf16 inputs, fp32 accumulation, the hidden activation rounded to bf16 once, y to bf16.
 *   x          in   bf16 [M][d]      grouped rows (slice-major, then local expert)
 *   offsets    in   int32 [S*E_loc + 1], non-decreasing, offsets[0] = 0, offsets[last] <= M
 *   w_gate,w_up in  [E_loc][f][d]    out-feature major (each output's d inputs contiguous)
 *   w_down     in   [E_loc][d][f]
 *   s_gate,s_up in  float [E_loc][f/128][d/128], s_down float [E_loc][d/128][f/128]
 *                   (MOE_W_FP8_E4M3_B128 only, else NULL): weight = decode(code) * scale
 *   y          out  bf16 [M][d]; rows >= offsets[last] are left untouched
 *   workspace       moe_ffn_workspace_bytes(M, d, f) bytes (holds the hidden activations).  With
 *                   MOE_W_FP8_E4M3_B128 the caller may add moe_ffn_expanded_weights_bytes(E_loc, d, f)
 *                   bytes: when there are at least 2048 rows per local expert on average the weights
 *                   are then expanded to bf16 once per call (the same values the kernels would form
 *                   tile by tile) and the faster bf16 kernels run
 * Limits: d % 256 == 0, f % 128 == 0, S*E_loc <= 65536, M < 2^31, d and f <= 2^22, d*f < 2^31
 * (MOE_ERR_UNSUPPORTED_SHAPE otherwise; M*d may exceed 2^31: rows are addressed with 64 bits); x, y,
 * the weights and the workspace 16-byte aligned (MOE_ERR_INVALID_ARG otherwise).  The sigmoid inside
 * silu uses the hardware reciprocal (within 1 ulp of the quotient, before the rounding to bf16).
 * ------------------------------------------------------------------------------------------- */
size_t     moe_ffn_workspace_bytes(int M, int d, int f);
size_t     moe_ffn_expanded_weights_bytes(int E_loc, int d, int f);
moe_status moe_expert_ffn_sliced(const void* x, const int32_t* offsets, int M, int S, int E_loc,
                                 int d, int f, int weight_format,
                                 const void* w_gate, const void* w_up, const void* w_down,
                                 const float* s_gate, const float* s_up, const float* s_down,
                                 void* y, void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * moe_expert_ffn_sliced_mapped -- moe_expert_ffn_sliced with the dispatch gather and the combine
 * scatter fused into the kernels (Section 2.1: dispatch / compute / combine): schedule row m reads
 * x[row_map[m]] (the gather happens in the copy that stages the operand tile) and its result goes
 * to y[row_map[m]], multiplied by row_gate[m] (the router weight of that (token, expert) pair) in
 * fp32 before the rounding to bf16:
 *     y[row_map[m]] = row_gate[m] * ( silu(x[row_map[m]] Wg_e^T) * (x[row_map[m]] Wu_e^T) ) Wd_e^T
 *   row_map    in   int32 [offsets[last]], a permutation of 0 .. offsets[last]-1 (e.g. row_arrival
 *                   of moe_slice_table_rows); NULL = identity
 *   row_gate   in   float [offsets[last]]; NULL = 1
 *   x, y            bf16 [M][d] in arrival order
 * Everything else as moe_expert_ffn_sliced.  Values of row_map outside [0, M) are not checked.
 * ------------------------------------------------------------------------------------------- */
moe_status moe_expert_ffn_sliced_mapped(const void* x, const int32_t* offsets, int M, int S, int E_loc,
                                        int d, int f, int weight_format,
                                        const void* w_gate, const void* w_up, const void* w_down,
                                        const float* s_gate, const float* s_up, const float* s_down,
                                        const int32_t* row_map, const float* row_gate,
                                        void* y, void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * moe_expert_ffn_backward_sliced -- Section 2.1: in training the dispatch -> compute -> combine
 * exchange is repeated for the gradients (the backward pass doubles the all-to-alls of a layer), so
 * the receiving rank also runs its experts backwards on the rows of every slice.  With
 * g = x Wg_e^T, u = x Wu_e^T, s = silu(g), h = s * u (the forward pass of moe_expert_ffn_sliced)
 * and dy the gradient with respect to y, for every row m of every group:
 *     dh = dy Wd_e ;  du = dh * s ;  dg = dh * u * silu'(g),  silu'(z) = sig(z) (1 + z (1 - sig(z)))
 *     dx[m] = dg Wg_e + du Wu_e
 * and for every local expert e, summed over its rows in all slices:
 *     dw_down[e] = dy^T h  [d][f] ;  dw_gate[e] = dg^T x  [f][d] ;  dw_up[e] = du^T x  [f][d]
 * bf16 inputs, fp32 accumulation; dh, dg, du and h are rounded to bf16 once (g and u are recomputed
 * from x, nothing is kept from the forward call), the outputs are bf16.
 *   x, dy      in   bf16 [M][d]   grouped rows as in moe_expert_ffn_sliced
 *   offsets    in   int32 [S*E_loc + 1]
 *   w_gate, w_up in bf16 [E_loc][f][d], w_down in bf16 [E_loc][d][f]   (bf16 weights only)
 *   dx         out  bf16 [M][d]; rows >= offsets[last] are left untouched
 *   dw_gate, dw_up out bf16 [E_loc][f][d], dw_down out bf16 [E_loc][d][f], overwritten (an expert
 *                   without rows gets zeros)
 *   workspace       moe_ffn_backward_workspace_bytes(M, E_loc, d, f) bytes
 * Limits: d % 256 == 0, f % 128 == 0, f >= 256, S*E_loc <= 65536, E_loc <= 4096, d*f < 2^30,
 * M < about 4 million rows (MOE_ERR_UNSUPPORTED_SHAPE otherwise); every pointer 16-byte aligned.
 * ------------------------------------------------------------------------------------------- */
size_t     moe_ffn_backward_workspace_bytes(int M, int E_loc, int d, int f);
moe_status moe_expert_ffn_backward_sliced(const void* x, const void* dy, const int32_t* offsets, int M, int S, int E_loc,
                                          int d, int f, const void* w_gate, const void* w_up, const void* w_down,
                                          void* dx, void* dw_gate, void* dw_up, void* dw_down,
                                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * moe_combine_topk_sum -- Section 2.1 (combine): the expert results travel back to the rank that
 * owns the tokens, where each token's output is the router-weighted sum over its topk experts:
 *     out[t] = sum_{j < topk} gate[t][j] * y[row_of[t][j]]
 * accumulated in fp32 in slot order j = 0, 1, ... (one fused multiply-add per term), rounded to bf16
 * once.
 *   y        in   bf16 [R][d]       expert results, one row per (token, expert) assignment, any order
 *   row_of   in   int32 [T][topk]   row of y that holds the result of token t's slot j; a value
 *                                   outside [0, R) (e.g. -1: dropped assignment) contributes nothing
 *   gate     in   float [T][topk]   router weights; NULL = 1 (e.g. when the weight was already applied
 *                                   by moe_expert_ffn_sliced_mapped's row_gate)
 *   out      out  bf16 [T][d], overwritten (a token with no live assignment gets zeros)
 * Limits: d % 8 == 0, T * topk < 2^31; y and out 16-byte aligned.  HBM bound: (topk + 1) * 2 * d
 * bytes per token.
 * ------------------------------------------------------------------------------------------- */
moe_status moe_combine_topk_sum(const void* y, const int32_t* row_of, const float* gate, int T, int topk, int d,
                                int R, void* out, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * moe_ffn_tile_override -- test and measurement hook, not meant for production callers.  The FFN
 * calls choose the height of their row blocks (64, 128 or 256 rows), the kernel family (one
 * whose tile shape adapts to ragged group ends, or fixed-shape tiles) and the order in which the
 * output tiles are walked from the shape of the schedule; this call pins any of these choices for
 * all following moe_expert_ffn_sliced(_mapped) calls of the process, so that every kernel can be
 * driven on small inputs and timed on any input.
 *   tile_rows    0 = chosen per call (the default), else 64, 128 or 256
 *   kernels      0 = chosen per call (the default), 1 = always the fixed-shape kernels, 2 = the
 *                adaptive-shape kernels with one launch per phase instead of both phases in one
 *                launch (where the adaptive-shape kernels apply)
 *   panel_groups 0 = chosen per call (the default), else the number of column groups (of up to 8
 *                column tiles) the tile walk finishes for all rows before it moves on to the next
 *                columns (a large value = all columns in one sweep per row group)
 * Process-wide and not synchronised with FFN calls running on other threads.  Results of any
 * choice agree within the rounding of the fp32 sums (the order of the additions differs).
 * Returns MOE_ERR_INVALID_ARG for other values (nothing changes then).
 * ------------------------------------------------------------------------------------------- */
moe_status moe_ffn_tile_override(int tile_rows, int kernels, int panel_groups);

/* ---------------------------------------------------------------------------------------------
 * moe_makespan_model -- Section 5 (Setup: "Execution time"), host-side.  Analytic completion time
 * of one MoE layer (dispatch -> expert compute -> combine on all N ranks) under a circuit schedule:
 * a matching occupies the network for reconf_s + duration * bytes_per_row / bandwidth (its largest
 * transfer over the link bandwidth); a rank starts the rows of matching i when that dispatch has
 * ended (and its previous rows are done) while the next dispatch proceeds; combine sends results
 * back over the same pairs.  Conventions where the paper's simulator is not specified: matching t
 * ships min(remaining entry, duration[t]) per pair; local rows (the diagonal) need no circuit and
 * are computed first; what the schedule leaves is served as one round lasting (largest line sum of
 * the residual) * bytes_per_row / bandwidth; the network serves all dispatches in order, then the
 * combines in order, each once every rank has finished that slice.
 * ALL POINTERS ARE HOST POINTERS; nothing is enqueued on the GPU.
 *   traffic     in  int32 [N][N]  communication matrix (row = source), diagonal = local rows
 *   perms       in  uint8 [K][N]  perms[t][i] = destination of source i in matching t
 *   durations   in  int32 [K]     hold time of matching t in rows
 *   order       in  int32 [K] or NULL: the matchings are played in this order (a permutation of
 *                   0..K-1); amounts shipped are those of the original order
 *   cost        in  see moe_cost_model
 *   out         out double [MOE_MAKESPAN_FIELDS] seconds:
 *                   [0] no overlap (every phase strictly after the other)   [1] with overlap
 *                   [2] idealised congestion-free all-to-all, no overlap      [3] sum of network phases (one way)
 *                   [4] sum over slices of the slowest rank's compute time
 * moe_order_matchings -- Section 4 (ordering the matchings as a flow-shop problem): Johnson's rule
 * for the two stages dispatch -> compute; writes the order into order_out int32 [K] (host).
 * Errors: MOE_ERR_INVALID_ARG (NULL, N < 1, K < 0, bad cost model, order not a permutation),
 * MOE_ERR_UNSUPPORTED_SHAPE (N > 256).
 * ------------------------------------------------------------------------------------------- */
#define MOE_COST_LINEAR 0   /* seconds = fixed_s + per_row_s * rows                                  */
#define MOE_COST_TABLE  1   /* measured (rows, seconds) points, rows ascending; linear in between,
                               the first point's time below it, the last segment continued above */
#define MOE_MAKESPAN_FIELDS 5
typedef struct moe_cost_model {
    double bytes_per_row;    /* bytes a (token, expert) row occupies on the wire, e.g. 2 * d          */
    double bandwidth;        /* bytes per second of one circuit                                       */
    double reconf_s;         /* reconfiguration delay per change of matching, seconds                 */
    int    kind;             /* MOE_COST_LINEAR or MOE_COST_TABLE; zero rows always cost nothing       */
    double fixed_s, per_row_s;
    const double* table_rows;     /* host [table_len] */
    const double* table_seconds;  /* host [table_len] */
    int    table_len;        /* >= 2 for MOE_COST_TABLE */
} moe_cost_model;

moe_status moe_makespan_model(const int32_t* traffic, int N, const uint8_t* perms, const int32_t* durations, int K,
                              const int32_t* order, const moe_cost_model* cost, double* out);
moe_status moe_order_matchings(const int32_t* traffic, int N, const uint8_t* perms, const int32_t* durations, int K,
                               const moe_cost_model* cost, int32_t* order_out);

/* ---------------------------------------------------------------------------------------------
 * moe_probe_mfma_bf16 -- measurement aid, not meant for production callers: the rate the matrix
 * cores sustain on v_mfma_f32_32x32x16_bf16 (the instruction of the expert FFN) from registers
 * alone, i.e. the ceiling of a bf16 contraction on this chip at the clock its power limit allows.
 * Enqueues one kernel of `workgroups` workgroups of four wavefronts; every wavefront issues
 * 16 * iters instructions of 32768 flop each, so the launch performs
 * workgroups * 4 * iters * 16 * 32768 flop; time it with the kernel timing below
 * ("mfma_probe_kernel") or with events of the caller.
 *   data        0 = all operands zero, 1 = operands drawn like the FFN's (about N(0,1) times
 *               N(0,0.02)); the sustained clock depends on it
 *   iters       1 .. 2^22
 *   workgroups  1 .. 4096 (one per compute unit fills the chip)
 *   sink        out  float [workgroups * 256]  one accumulator per thread (keeps the loop alive)
 * ------------------------------------------------------------------------------------------- */
moe_status moe_probe_mfma_bf16(int data, int iters, int workgroups, float* sink, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * Kernel timing (measurement aid).  While enabled, every kernel launch of this library is
 * bracketed by HIP events on the caller's stream.  moe_kernel_timing_read synchronises those
 * events, adds them up per kernel name and resets the table.
 *   names  host out  up to `cap` pointers to static strings
 *   total_ms, launches  host out  summed duration and number of launches per name
 * Returns the number of distinct kernel names (<= cap) or a negative moe_status.
 * Not thread safe; intended for single-threaded benchmarks.
 * ------------------------------------------------------------------------------------------- */
moe_status moe_kernel_timing_enable(int on);
/* Restrict the timing to one kernel name (as reported by moe_kernel_timing_read, e.g. "ffn_gemm1_kernel"; host
 * string, copied): an event pair costs a few microseconds of stream time, which matters when a whole step of
 * small kernels is being measured at the same time.  NULL = every kernel (the default). */
moe_status moe_kernel_timing_select(const char* kernel_name);
int        moe_kernel_timing_read(const char** names, float* total_ms, int* launches, int cap);

/* Text of the last HIP error seen by this library in the calling process (host pointer). */
const char* moe_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MOE_CIRCUIT_H */

/*
 * moegps.h -- C ABI of libmoegps: one MoE FFN layer with dynamic expert
 * duplication (the setting of MoE-GPS, arXiv 2506.07366) on one AMD MI355X.
 *
 * The layer is split into the calls of the paper's problem statement: gate
 * top-k routing, the per-expert token histogram that Distribution-Only
 * Prediction forecasts (Eq. (1)), the duplication plan (Algorithm 1), the
 * dispatch/permutation of tokens to replicas, the grouped SwiGLU expert FFN and
 * the weighted combine.  G expert-parallel ranks with S expert slots each are
 * emulated as partitions of one GPU; a "segment" is one slot, global id g*S+s.
 *
 * Conventions for every call
 *   - Every pointer is a DEVICE pointer unless it is marked "host".  Buffers are
 *     contiguous, row-major, 16-byte aligned and owned by the caller; the
 *     library never allocates, frees or keeps device memory.  Scratch space is
 *     passed in as a workspace whose size comes from a *_workspace_bytes query.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue kernels on it and return; there is no host
 *     synchronisation inside, results are valid in stream order.
 *   - Return value: MOE_OK (0) or a negative MOE_ERR_* code.  Arguments are
 *     checked on the host (scalars and NULL pointers only); on an error nothing
 *     has been enqueued.  No exception or abort crosses the boundary.
 *   - dtype: MOE_DTYPE_F32 (float) or MOE_DTYPE_BF16 (bfloat16 storage, fp32
 *     accumulation).
 *   - Notation: T tokens, E experts, k experts per token, A = T*k assignments
 *     (assignment a = t*k + j is token t's j-th expert), d model width, ffn
 *     expert hidden width, G ranks, S slots per rank, NSEG = G*S.
 */
#ifndef MOEGPS_H
#define MOEGPS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_OK                        0
#define MOE_ERR_INVALID_ARG         (-1)
#define MOE_ERR_UNSUPPORTED         (-2)   /* shape or dtype outside what is built */
#define MOE_ERR_WORKSPACE_TOO_SMALL (-3)
#define MOE_ERR_HIP                 (-4)   /* a HIP call failed, see moe_last_hip_error */

#define MOE_DTYPE_F32   0
#define MOE_DTYPE_BF16  1

#define MOE_MODE_NONE          0   /* home placement only (no prediction) */
#define MOE_MODE_DISTRIBUTION  1   /* Distribution-Only Prediction, Section 3.2.1 */
#define MOE_MODE_TOKEN         2   /* Token-to-Expert Prediction, Section 3.2.2 */

/* compile-time limits of the library */
#define MOE_MAX_EXPERTS   1024
#define MOE_MAX_TOPK        16
#define MOE_MAX_RANKS      256
#define MOE_MAX_SLOTS       16   /* per rank */
#define MOE_MAX_SEGMENTS  2048   /* G*S */

/* Text for a return code (host pointer to a static string). */
const char* moe_strerror(int code);
/* The hipError_t (as int) recorded by the last call that returned MOE_ERR_HIP on this thread. */
int moe_last_hip_error(void);
/* Version of this ABI (increases when a signature changes). */
int moe_abi_version(void);

/*
 * Gate top-k (Background: each token is routed to its top-K experts; the
 * token->expert map f of Algorithm 1).
 *   logits   [T, E] float  in   router logits, given directly (finite values)
 *   topk_idx [T, k] int32  out  experts ordered by (logit descending, index
 *                               ascending): equal logits go to the lowest index
 *   topk_w   [T, k] float  out  softmax over the k selected logits
 * 1 <= k <= min(E, MOE_MAX_TOPK), E <= MOE_MAX_EXPERTS.  T = 0 is a no-op.
 */
int moe_route_topk(const float* logits, int T, int E, int k,
                   int32_t* topk_idx, float* topk_w, void* stream);

/*
 * Per-expert count n_e = #{a : idx[a] == e} (the n_i of Eq. (1); p_hat_i = n_i/N).
 *   idx  [n] int32 in   values in [0, E); values outside are ignored
 *   hist [E] int32 out  overwritten (not accumulated)
 */
int moe_histogram(const int32_t* idx, int64_t n, int E, int32_t* hist, void* stream);

/*
 * Expert duplication plan (Algorithm 1, count-based).  Starts from the home
 * placement (expert e on rank e / H, slot e % H, H = ceil(E/G)) with every
 * predicted token on its home, then repeats: hottest rank g_h, coldest rank
 * g_c, Delta = ceil((L_h - L_c)/2), hottest expert e* on g_h; replicate e* into
 * the lowest empty slot of g_c if it is not there, has fewer than c_max copies
 * and g_c has room; move min(Delta, tokens of e* on g_h) tokens.  If that
 * candidate is infeasible the next experts of g_h (descending load) and then the
 * next-coldest ranks are tried; the loop ends when max L - min L <= 1, nothing is
 * feasible, or after 16*G*S iterations.  All ties go to the lowest index.
 *   mode            MOE_MODE_NONE stops after the home placement
 *   hist_pred [E]   int32 in   predicted counts (mode 2: histogram of the
 *                              predicted ids, computed by the caller with
 *                              moe_histogram); must be >= 0
 *   c_max           max copies of one expert (>= 1)
 *   slot_expert    [G*S] int32 out  expert hosted by each slot, -1 = empty
 *   slot_quota     [G*S] int32 out  planned rows per slot
 *   rank_load_pred [G]   int32 out  planned rows per rank
 *   n_iters        [1]   int32 out  iterations of the loop that moved tokens
 * Requires ceil(E/G) <= S <= MOE_MAX_SLOTS, G <= MOE_MAX_RANKS.
 */
int moe_plan_duplicates(int mode, const int32_t* hist_pred, int E, int G, int S, int c_max,
                        int32_t* slot_expert, int32_t* slot_quota, int32_t* rank_load_pred,
                        int32_t* n_iters, void* stream);

/*
 * Dispatch + permutation (the dispatch d of Algorithm 1; stands where the
 * all-to-all before the expert FFN is; Background, paragraph on the communication
 * cost of routing).  Every assignment gets a segment:
 *   mode 0: the home slot of its expert;
 *   mode 1: replicas of expert e in ascending slot id take contiguous ranges of
 *           e's assignments (ascending a) with boundaries floor(n_e*Q_r/nhat_e),
 *           Q_r = cumulative planned quota; nhat_e = 0 -> home slot;
 *   mode 2: if the true expert is among the token's predicted ids, the
 *           assignment takes its place (stable rank among predicted assignments
 *           of e) in the planned quotas; otherwise it falls back to the home slot
 *           of its true expert.
 * Then the assignments are sorted stably by segment and rows are copied.
 *   x          [T, d]  dtype in
 *   topk_idx   [T, k]  int32 in
 *   pred_idx   [T, k]  int32 in   mode 2 only (rows hold distinct ids), else NULL
 *   hist_true  [E]     int32 in   histogram of topk_idx (mode 1)
 *   hist_pred  [E]     int32 in   the histogram the plan was built from (mode 1)
 *   slot_expert, slot_quota [G*S] int32 in   the plan
 *   seg_offsets   [G*S+1] int32 out  first row of each segment, last = A
 *   row_of_assign [A]     int32 out  row of x_perm that holds assignment a
 *   assign_of_row [A]     int32 out  inverse permutation
 *   x_perm        [A, d]  dtype out  x_perm[row] = x[assign_of_row[row] / k]; may be
 *                                    NULL to skip the row copy
 *   rank_load     [G]     int32 out  rows served by each rank
 * d * sizeof(dtype) must be a multiple of 16.  A < 2^31.  The size query returns 0 for
 * arguments outside the limits above (MOE_MAX_*).
 */
size_t moe_permute_workspace_bytes(int T, int E, int k, int G, int S);
int moe_permute(int mode, const void* x, int dtype, int T, int d, int E, int k, int G, int S,
                const int32_t* topk_idx, const int32_t* pred_idx,
                const int32_t* hist_true, const int32_t* hist_pred,
                const int32_t* slot_expert, const int32_t* slot_quota,
                int32_t* seg_offsets, int32_t* row_of_assign, int32_t* assign_of_row,
                void* x_perm, int32_t* rank_load,
                void* workspace, size_t workspace_bytes, void* stream);

/*
 * moe_permute for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation.  Arguments, outputs
 * and limits are those of moe_permute without `workspace`/`workspace_bytes`; the counters,
 * chunk bases and segment ids live in a fixed array of MOE_PERMUTE_STATIC_SCRATCH_BYTES that
 * the library keeps in device memory (every GPU the library runs on holds its own copy until
 * the process ends).  The call allocates nothing and runs the same kernels, so its outputs are
 * bit-identical to moe_permute's.  Sizes with
 *     moe_permute_workspace_bytes(T, E, k, G, S) > MOE_PERMUTE_STATIC_SCRATCH_BYTES
 * are refused with MOE_ERR_WORKSPACE_TOO_SMALL before anything is enqueued (8 MiB holds about
 * 1.8 million assignments at 128 experts and 160 segments).  All calls on one GPU share that GPU's array, and
 * nothing in it needs clearing between calls (every entry a call reads it has written first);
 * calls that overlap on one GPU -- two streams, two host threads -- race on it: serialise them.
 */
#define MOE_PERMUTE_STATIC_SCRATCH_BYTES (8u << 20)
int moe_permute_static(int mode, const void* x, int dtype, int T, int d, int E, int k, int G, int S,
                       const int32_t* topk_idx, const int32_t* pred_idx,
                       const int32_t* hist_true, const int32_t* hist_pred,
                       const int32_t* slot_expert, const int32_t* slot_quota,
                       int32_t* seg_offsets, int32_t* row_of_assign, int32_t* assign_of_row,
                       void* x_perm, int32_t* rank_load, void* stream);

/*
 * One-off repack of the expert weights into the tile order the FFN kernels
 * stream (expert weights are static across inputs, Discussion "Expert
 * duplication's communication overhead"; not part of the per-batch path).
 *   W1, W3 [E, d, ffn], W2 [E, ffn, d]  dtype in (row-major)
 *   packed  out, moe_packed_weights_bytes(E, d, ffn, dtype) bytes
 * For MOE_DTYPE_F32 the packed form is a plain copy.  For MOE_DTYPE_BF16 every matrix is
 * stored transposed, in tiles of 256 output columns by 64 of the contracted dimension,
 * each tile 32 KiB in one piece in the order the kernels hold it on chip; the hidden width
 * is padded to a multiple of 64 and the output columns to whole tiles with zeros (the
 * size query includes the padding).  The packed form is opaque: only these calls read it.
 */
size_t moe_packed_weights_bytes(int E, int d, int ffn, int dtype);
int moe_pack_weights(const void* W1, const void* W3, const void* W2, int dtype,
                     int E, int d, int ffn, void* packed, void* stream);

/*
 * Grouped SwiGLU expert FFN (Section 3.4: Mixtral-style FFN with SwiGLU; the
 * dominant cost of the layer, Background "Performance Impacts").  For every row
 * r of a segment sigma in [seg_begin, seg_end) with e = slot_expert[sigma]:
 *     y_perm[r] = ( silu(x_perm[r] W1_e) * (x_perm[r] W3_e) ) W2_e
 * Rows of other segments are not written.  seg_begin/seg_end select a slot
 * range, e.g. one rank's [g*S, (g+1)*S), so a rank's share can be timed alone.
 *   x_perm [A, d] dtype in;  y_perm [A, d] dtype out
 *   seg_offsets [nseg+1], slot_expert [nseg] int32 in (device; read by the kernels)
 *   packed  in  weights from moe_pack_weights
 * Rows are tiled by expert: the rows of all segments of the range that host one expert are
 * multiplied under that expert's weight panels together (replicas hold the same weights), so
 * the result of a row depends on its values and its expert only.
 * bf16: products accumulate in fp32, the hidden activation is rounded to bf16 between the
 * two products, the output is rounded to bf16.  SwiGLU uses the hardware exponential and
 * reciprocal instructions (about 1 ulp each, far below the bf16 rounding that follows).
 * When the second product has only a few tiles per workgroup, its closing tiles are summed as
 * up to four parts of the hidden width (fp32 partial sums held in the workspace, added in the
 * order of the parts, then rounded once); the result does not depend on launch order.
 * bf16 needs d % 64 == 0 (any ffn: the packed weights pad the hidden width to a multiple of
 * 64 with zeros) and A * d < 2^31; f32 needs d % 4 == 0 and ffn % 4 == 0.
 * Limits: 0 <= A < 2^31, 1 <= d, ffn <= 2^22, 1 <= nseg <= MOE_MAX_SEGMENTS.  The size query
 * returns 0 for arguments outside them (every size query of this library does).
 */
size_t moe_grouped_ffn_workspace_bytes(int64_t A, int d, int ffn, int nseg, int dtype);
int moe_grouped_ffn(const void* x_perm, int dtype, int64_t A, int d, int ffn, int E,
                    const int32_t* seg_offsets, const int32_t* slot_expert, int nseg,
                    int seg_begin, int seg_end, const void* packed,
                    void* y_perm, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Same FFN with the boundary copies folded in.  The activation rows are gathered inside the
 * first product instead of being read from a permuted copy: row r of the (virtual) x_perm is
 * x[assign_of_row[r] / k], so moe_permute can be called with x_perm = NULL, which removes one
 * write and one read of A*d elements from the layer.  With topk_w != NULL the second product
 * also multiplies row r of its result by the gate weight of its assignment,
 * topk_w[assign_of_row[r]], in fp32 before the row is rounded; moe_combine is then called with
 * topk_w = NULL and only adds the k rows of a token (the weighted sum of the return
 * all-to-all, Background, moved in front of the transfer).  moe_grouped_ffn_gather is the call
 * without gate weights: its output and numerics are those of moe_grouped_ffn on the copied rows.
 *   x [T, d] dtype in;  assign_of_row [T*k] int32 in (from moe_permute);
 *   topk_w [T, k] float in or NULL
 * The other arguments are those of moe_grouped_ffn with A = T*k.  T*d < 2^31.
 */
int moe_grouped_ffn_fused(const void* x, int dtype, int T, int k, const int32_t* assign_of_row,
                          const float* topk_w, int d, int ffn, int E,
                          const int32_t* seg_offsets, const int32_t* slot_expert, int nseg,
                          int seg_begin, int seg_end, const void* packed,
                          void* y_perm, void* workspace, size_t workspace_bytes, void* stream);
int moe_grouped_ffn_gather(const void* x, int dtype, int T, int k, const int32_t* assign_of_row,
                           int d, int ffn, int E,
                           const int32_t* seg_offsets, const int32_t* slot_expert, int nseg,
                           int seg_begin, int seg_end, const void* packed,
                           void* y_perm, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Overrides of the automatic choices inside the grouped FFN, for tests and experiments
 * (process-wide; set them before sizing a workspace, the split option changes its size):
 *   MOE_FFN_OPT_TILE1 / TILE2  tile shape of the first / second product: -1 automatic,
 *                              0 = 256x256x64, 1 = 128x256x64, 2 = 32x256x64
 *   MOE_FFN_OPT_SPLIT_K        closing tiles of the second product as parts of K:
 *                              -1 automatic, 0 never, 1 whenever the shapes allow
 *   MOE_FFN_OPT_GROUP_N        N-tiles walked side by side under one run of M-tiles, 0 automatic
 * Returns MOE_ERR_INVALID_ARG for an unknown option or a value out of range.
 */
#define MOE_FFN_OPT_TILE1    0
#define MOE_FFN_OPT_TILE2    1
#define MOE_FFN_OPT_SPLIT_K  2
#define MOE_FFN_OPT_GROUP_N  3
int moe_grouped_ffn_set_option(int option, int value);

/*
 * The ReLU form of the expert FFN (Discussion, "Generality across model architectures":
 * Switch Transformer uses ReLU in its FFN, with top-1 routing):
 *     y_perm[r] = max(x_perm[r] W1_e, 0) W2_e        no gate matrix, no biases
 * moe_pack_weights_relu repacks W1 [E, d, ffn] and W2 [E, ffn, d] into
 * moe_packed_weights_relu_bytes(E, d, ffn, dtype) bytes; moe_grouped_ffn_relu takes the
 * arguments of moe_grouped_ffn (same workspace size, same limits, same precision rules:
 * bf16 storage, fp32 accumulation, the hidden activation rounded to bf16) with that
 * packed buffer.
 */
size_t moe_packed_weights_relu_bytes(int E, int d, int ffn, int dtype);
int moe_pack_weights_relu(const void* W1, const void* W2, int dtype,
                          int E, int d, int ffn, void* packed, void* stream);
int moe_grouped_ffn_relu(const void* x_perm, int dtype, int64_t A, int d, int ffn, int E,
                         const int32_t* seg_offsets, const int32_t* slot_expert, int nseg,
                         int seg_begin, int seg_end, const void* packed,
                         void* y_perm, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Optional timing hook for the next moe_grouped_ffn* call on this host thread:
 * events[0..3] are hipEvent_t handles (as void*) that the call records on its
 * stream before and after its first product (gate/up + SwiGLU) and before and
 * after its second product (down).  The hook is consumed by that one call, also when the
 * call returns early or takes the fp32 path (which records nothing).
 * Pass NULL to clear it.  `events` is a HOST array of 4 handles; it is copied.
 */
int moe_grouped_ffn_time_next_call(void* const* events);

/*
 * Weighted un-permute (stands where the all-to-all after the FFN is):
 *     out[t, :] = sum_{j<k} topk_w[t, j] * y_perm[row_of_assign[t*k + j], :]
 * summed in fp32 with j ascending; bf16 output is rounded once at the end.
 *   y_perm [A, d] dtype in, row_of_assign [A] int32 in, topk_w [T, k] float in,
 *   out [T, d] dtype out.  d * sizeof(dtype) must be a multiple of 16.
 * topk_w = NULL adds the k rows unweighted (rows that moe_grouped_ffn_fused has already
 * multiplied by their gate weights).
 */
int moe_combine(const void* y_perm, int dtype, int T, int d, int k,
                const int32_t* row_of_assign, const float* topk_w, void* out, void* stream);

/*
 * Rows that cross the emulated expert-parallel ranks (Background, paragraph on the
 * communication cost of routing: with N ranks and a balanced distribution (N-1)/N of a
 * rank's rows leave it and the rank of the most popular expert receives skewness times
 * the average; the all-to-all after the FFN moves the same rows back.  Section 3.2.2:
 * under Token-to-Expert prediction a correctly predicted token is already on the rank of
 * its expert; Section 3.3: a mispredicted one still has to be moved).
 * Token t is owned by rank floor(t*G/T).  For every assignment a = t*k + j, with
 * dst = rank of the segment that holds row_of_assign[a]:
 *     dispatch[src*G + dst] += 1   src = owner(t), or dst when mode is MOE_MODE_TOKEN and
 *                                  topk_idx[a] is among pred_idx[t, 0..k)
 *     combine[dst*G + owner(t)] += 1
 *   topk_idx [T, k], pred_idx [T, k] (MOE_MODE_TOKEN only, else may be NULL),
 *   row_of_assign [A], seg_offsets [G*S + 1] (outputs of moe_permute): device in;
 *   dispatch, combine [G, G] int32: device out, overwritten (all zero when T = 0).
 * Limits as for moe_permute.  Returns MOE_ERR_INVALID_ARG / MOE_ERR_UNSUPPORTED before
 * any launch when an argument is out of range.
 */
int moe_comm_matrix(int mode, int T, int k, int G, int S,
                    const int32_t* topk_idx, const int32_t* pred_idx,
                    const int32_t* row_of_assign, const int32_t* seg_offsets,
                    int32_t* dispatch, int32_t* combine, void* stream);

/*
 * Distribution-Only predictor (Section 3.2.1, Eq. (1); Appendix A): the maximum-likelihood
 * estimate of a layer's expert distribution is p_hat_i = n_i / N over all tokens seen so
 * far (a running average when the data come in batches).
 *   moe_predictor_update : counts[e] += hist[e]          (hist: one batch's moe_histogram)
 *   moe_predictor_predict: hist_pred = p_hat * A_next brought to integers that sum to
 *                          A_next by largest remainder (ties -> lowest expert); uniform
 *                          while nothing has been seen (all counts zero).
 *   hist [E] int32 device in; counts [E] int64 device in/out, owned and zeroed by the caller
 *   before the first batch, total below 2^62; hist_pred [E] int32 device out, a valid
 *   `hist_pred` for moe_plan_duplicates / moe_permute in MOE_MODE_DISTRIBUTION.
 * E <= MOE_MAX_EXPERTS, 0 <= A_next < 2^31.  Exact integer arithmetic.
 */
int moe_predictor_update(const int32_t* hist, int E, int64_t* counts, void* stream);
int moe_predictor_predict(const int64_t* counts, int E, int64_t A_next, int32_t* hist_pred, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOEGPS_H */

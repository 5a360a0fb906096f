/*
 * zr.h - C ABI of the MI355X (gfx950) library for one tensor-parallel task's
 *        resized shard GEMMs (ZERO-resizing, arXiv 2401.11469, Sec. 3).
 *
 * A straggling task prunes a priority-selected subset of one axis of its
 * weight shard for one step, multiplies what is left (forward, dX, dW), and
 * recovers the normal shape of every output by imputing the missing slices
 * (Sec. 3.1 "Overview Resizing Design", "Consistency Constraint").
 *
 * Notation.  M = tokens (bs*sql).  X[M x K] activations, W[K x N] weight shard
 * (in-features x out-features), Y[M x N] = X W, dY[M x N], dX[M x K] = dY W^T,
 * dW[K x N] = X^T dY.  The paper stores weight as [out, in]; its "columns of
 * input and weight" are axis K here.
 *
 * General conventions
 *  - Every tensor / index pointer is a DEVICE pointer owned by the caller.  The
 *    library allocates nothing, frees nothing and keeps no state between calls
 *    (zr_debug.h declares optional measuring aids that do keep a little).
 *  - Tensors are row-major; leading dimensions (ld*) are in ELEMENTS and must be
 *    >= the row length.  bf16 tensors whose base is 16-byte aligned and whose
 *    ld is a multiple of 8 (fp32: 4) take the vectorised paths; anything else is
 *    still computed correctly on an element-wise path.
 *  - Every call only enqueues work on `stream` (a hipStream_t passed as void*;
 *    NULL = the default stream) and never synchronises, except
 *    zr_validate_keep_idx, which is a debugging aid.
 *  - Errors are return codes; no call aborts or throws.  Every argument check
 *    happens before the first launch: on NULL, SHAPE, RATIO, INDEX, DTYPE, MODE,
 *    POLICY and LIMIT nothing is enqueued and the outputs are untouched.  Only
 *    ZR_ERR_HIP (the runtime refused a launch) can come after earlier kernels of
 *    the same call were enqueued; the outputs are then undefined.
 *  - Calls may be made from several host threads (the library keeps no state
 *    between calls; the aids of zr_debug.h are per thread).
 *  - keep_idx is the kept index set: int32, strictly ascending, unique, within
 *    [0, n) of the pruned axis.  It plays the role of the paper's lineage
 *    tuple: the same list is shared by input and weight (Sec. 3.2) and reused
 *    from forward to backward.  A list violating this gives undefined OUTPUT
 *    VALUES but never an out-of-range access: indices are clamped into range.
 *  - Accumulation is always fp32; outputs have the input dtype.  Kept
 *    contributions are not rescaled (outputs just miss the pruned partial
 *    products, Sec. 3.2 first paragraph).
 */
#ifndef ZR_H
#define ZR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ZR_OK = 0,
    ZR_ERR_NULL = 1,      /* a required pointer is NULL */
    ZR_ERR_SHAPE = 2,     /* a size is negative/zero where it may not be, or ld < row length */
    ZR_ERR_RATIO = 3,     /* ratio outside [0,1) or it leaves no kept index */
    ZR_ERR_INDEX = 4,     /* n_keep outside [1, n] (or, from the validator, a bad list) */
    ZR_ERR_DTYPE = 5,
    ZR_ERR_MODE = 6,
    ZR_ERR_POLICY = 7,    /* unknown policy, or SAME without the previous tensor */
    ZR_ERR_LIMIT = 8,     /* size beyond what the kernels index (M, K, N or rows above 65535 * 32; see each call) */
    ZR_ERR_HIP = 9        /* a HIP runtime call failed (launch error) */
} zr_status;

typedef enum { ZR_F32 = 0, ZR_BF16 = 1 } zr_dtype;

/* Which axis of W[K x N] keep_idx indexes.
 *  ZR_DROP_K: the contraction axis (the paper's worked example, and the reading
 *             used for row-parallel shards): Y keeps its shape and misses
 *             partial products; dX loses columns, dW loses rows -> imputed.
 *  ZR_DROP_N: the output-feature axis (the dual case, used for column-parallel
 *             shards): Y and dW lose columns -> imputed; dX keeps its shape. */
typedef enum { ZR_DROP_N = 0, ZR_DROP_K = 1 } zr_mode;

/* How the weight shard (and its gradient) is stored.
 *  ZR_W_KN: W[K x N] row-major ([in, out]); ldw >= N.
 *  ZR_W_NK: the transpose, [N x K] row-major ([out, in], the layout of the
 *           paper's weight matrix, Sec. 3.1); ldw >= K.
 * The mathematics is the same; the layout decides whether the kept list selects
 * ROWS of the stored matrix (contiguous: gathered while the tiles are loaded,
 * the weight is never copied) or single elements of every row (slower loaders).
 * Rows are selected for (ZR_W_KN, ZR_DROP_K) and (ZR_W_NK, ZR_DROP_N): store
 * row-parallel shards as KN and column-parallel shards as NK. */
typedef enum { ZR_W_KN = 0, ZR_W_NK = 1 } zr_w_layout;

/* Flags of the backward call's workspace.
 *  ZR_WS_HOLDS_FORWARD: the buffer is the one the forward call of the SAME layer
 *  step was given (same X, keep_idx, sizes, mode, dtype) and nothing has written
 *  to it since: what the forward extracted (X[:,S] in DROP_K) is used again
 *  instead of being extracted a second time; this is the pruned input that the
 *  paper's layer keeps for its backward pass (Sec. 3.1).  Without the flag the
 *  backward call extracts what it needs itself.  Results are identical. */
typedef enum { ZR_WS_FRESH = 0, ZR_WS_HOLDS_FORWARD = 1 } zr_ws_flags;

/* Imputation policies (Sec. 3.1, the paragraph on which value fills a pruned position). */
typedef enum {
    ZR_IMPUTE_ZERO = 0,     /* +0.0 (the paper's final choice) */
    ZR_IMPUTE_AVERAGE = 1,  /* element-wise mean of the kept slices of this result */
    ZR_IMPUTE_SAME = 2      /* value of the previous iteration's tensor at that position */
} zr_policy;

const char* zr_status_string(int status);

/* Kept count for a pruned axis of length n at pruning ratio gamma
 * (Algorithm 1: L_pri = L*(1-gamma)), rounded half-up in IEEE double:
 * floor((1-ratio)*n + 0.5).  Pure host function.  Returns -1 if n < 0 or ratio is
 * outside [0,1) (NaN included). */
int64_t zr_keep_count(int64_t n, double ratio);

/* Priority selection (Algorithm 1: top-L_pri select, then ascending sort).
 *  scores   [batch x n] fp32, row b at scores + b*n: importance of each index
 *           (larger = kept first).  NaN ranks lowest, -0.0 == +0.0, ties keep the
 *           lower index.
 *  keep_idx [batch x ld_idx] int32 out: row b receives the n' = zr_keep_count(n,
 *           ratio) kept indices, ascending.  ld_idx >= n'.
 *  drop_idx [batch x ld_idx] int32 out or NULL: the n - n' pruned indices,
 *           ascending (the set P of the lineage tuple).  ld_idx >= n - n' too.
 *  One launch; one workgroup per score vector.  n <= 2^24.
 *  Errors: NULL, SHAPE (n < 1, batch < 1, ld_idx too small), RATIO, LIMIT. */
int zr_resize_select(const float* scores, int32_t n, int32_t batch, double ratio,
                     int32_t* keep_idx, int32_t* drop_idx, int64_t ld_idx, void* stream);

/* The same selection for ONE long vector, spread over many workgroups (Alg. 1's
 * top-L_pri select at lengths far beyond a layer shard's, e.g. one list over
 * a whole model).  With a DEVICE scratch buffer of at least
 * zr_select_workspace_bytes(n) bytes (4-byte aligned; 68 KB) and n >= 131072
 * the vector is cut into slices of 4096 scores, one wavefront each: four
 * histogram launches (one per key byte), a count, a scan of the per-slice
 * counts and the ordered write, every launch reading the vector once; all
 * counters are integers, so the lists are the same, bit for bit, as
 * zr_resize_select's.  Shorter vectors, or a missing / too small buffer, take
 * zr_resize_select's single workgroup.  The buffer's contents are undefined
 * afterwards; calls that share one must be ordered on one stream.
 * zr_select_workspace_bytes: pure host function, 0 for n below the threshold.
 *  Errors: NULL, SHAPE (n < 1), RATIO, LIMIT (n > 2^24). */
size_t zr_select_workspace_bytes(int32_t n);
int zr_resize_select_ws(const float* scores, int32_t n, double ratio, int32_t* keep_idx, int32_t* drop_idx,
                        void* workspace, size_t workspace_bytes, void* stream);

/* The same selection for `count` (<= 16) independent score vectors of different
 * lengths in ONE launch, e.g. all projections of a layer shard at the start of
 * a step.  scores, n, ratio, keep_idx, drop_idx are HOST arrays of `count`
 * entries; scores[b], keep_idx[b], drop_idx[b] are DEVICE pointers (drop_idx, or
 * any drop_idx[b], may be NULL); keep_idx[b] holds zr_keep_count(n[b], ratio[b])
 * entries, drop_idx[b] the rest.  The host arrays are read before the call
 * returns.  Errors: NULL, SHAPE, RATIO, LIMIT (count > 16, n > 2^24). */
int zr_resize_select_multi(int32_t count, const float* const* scores, const int32_t* n, const double* ratio,
                           int32_t* const* keep_idx, int32_t* const* drop_idx, void* stream);

/* Size of the optional scratch buffer of the forward / backward calls below.
 * With a DEVICE buffer of at least this many bytes (16-byte aligned) the calls
 * first extract the kept columns of the ACTIVATION they would otherwise gather
 * along its contiguous axis (X[:,S] for DROP_K, dY[:,S] for DROP_N; the pruned
 * input of Sec. 3.1's forward paragraph) into it,
 * [M x n_keep rounded up to 64] bf16, zero padded, and then run the products on
 * ordinary loads.  The weight shard is never copied or compacted, in either
 * layout.  Without it (NULL, or too small) every gather is done in flight by
 * the GEMM loaders.
 * Layout: the extracted activation (bf16 only); then 64 MiB (bf16 only) for
 * the slices of a split contraction; then, at the tail (both dtypes), the
 * per-tile sums of ZR_IMPUTE_AVERAGE: the products' epilogues leave sums of
 * the stored results there, from which the means of the dropped slices are
 * taken; without it a second pass re-reads the kept slices (means equal up to
 * fp32 summation order).
 * Split contraction: a bf16 product (or remainder panel of one) that would
 * occupy fewer than half of the chip's compute units and whose contraction is
 * at least 1024 long is computed in 2..8 slices of the contraction in a first
 * launch (fp32 partial results in the buffer) and summed, slice after slice,
 * and stored by a second one.  Such a result differs from the one-launch result
 * by fp32 summation order (the element-wise bound of the output type still
 * holds); it is repeatable bit by bit for a given buffer size.  Results of
 * products that are not split are the same to the last bit with and without
 * the buffer.  A buffer smaller than this size is used as far as it reaches
 * (extraction first).  Pure host function; returns 0 on bad sizes. */
size_t zr_workspace_bytes(int32_t M, int32_t K, int32_t N, int32_t n_keep, int mode, int dtype);

/* The extraction step on its own (Sec. 3.1, forward paragraph: the kept columns
 * of the input, side by side in ascending index order): out[r, q] = in[r, keep_idx[q]] for
 * q < n_keep, and +0 for n_keep <= q < width, width = n_keep rounded up to 64.
 *  in [rows x n] ld, out [rows x width] ldo >= width; bf16 only (else DTYPE);
 *  ld, ldo and n even, in and out 4-byte aligned (else SHAPE).  One launch.
 * The forward / backward calls run exactly this kernel when given a workspace. */
int zr_extract_kept_columns(const void* in, int64_t ld, int32_t rows, int32_t n,
                            const int32_t* keep_idx, int32_t n_keep,
                            void* out, int64_t ldo, int dtype, void* stream);

/* Forward of the resized linear layer (Sec. 3.1, forward paragraph).
 *  DROP_K: Y = X[:,S] W[S,:]            (full shape, nothing to impute)
 *  DROP_N: Y[:,S] = X W[:,S];  Y[:,P] imputed by `policy`
 *  X [M x K] ldx, W stored per w_layout with ldw, Y [M x N] ldy (out, every
 *  element written).  keep_idx[n_keep] indexes K (DROP_K) or N (DROP_N).
 *  prev_Y: previous iteration's Y [M x N] with leading dimension ldy, needed for
 *  ZR_IMPUTE_SAME in DROP_N only (may alias Y: dropped positions then stay as
 *  they are); ignored otherwise.
 *  workspace / workspace_bytes: optional scratch, see zr_workspace_bytes; its
 *  contents are undefined afterwards; calls that share one must be ordered on
 *  one stream.
 *  Launches: 1 for ZERO and SAME (both written by the product's own epilogue),
 *  +1 with a workspace in DROP_K; AVERAGE: +1 (stand-alone pass) or +3 small ones
 *  (clear sums, means, fill) with a workspace.
 *  Errors: NULL, SHAPE, INDEX, DTYPE, MODE (also a bad w_layout), POLICY, LIMIT, HIP. */
int zr_resized_linear_fwd(const void* X, int64_t ldx, const void* W, int64_t ldw,
                          void* Y, int64_t ldy, int32_t M, int32_t K, int32_t N,
                          const int32_t* keep_idx, int32_t n_keep,
                          int mode, int w_layout, int dtype, int policy, const void* prev_Y,
                          void* workspace, size_t workspace_bytes, void* stream);

/* Backward of the resized linear layer (Sec. 3.1, backward paragraph; the
 * upstream gradient is never pruned in the paper's DROP_K case).
 *  DROP_K: dX[:,S] = dY W[S,:]^T, dX[:,P] imputed;  dW[S,:] = X[:,S]^T dY, dW[P,:] imputed
 *  DROP_N: dX = dY[:,S] W[:,S]^T (full shape);      dW[:,S] = X^T dY[:,S], dW[:,P] imputed
 *  dX [M x K] lddx and dW (stored like W: [K x N] or [N x K], lddw) are outputs;
 *  either may be NULL to skip that product.  prev_dX / prev_dW (same shapes,
 *  layout and leading dimensions as dX / dW) are read for ZR_IMPUTE_SAME only.
 *  workspace: as for the forward call; workspace_flags: see zr_ws_flags (0 = none).
 *  Errors as for the forward call. */
int zr_resized_linear_bwd(const void* X, int64_t ldx, const void* W, int64_t ldw,
                          const void* dY, int64_t lddy,
                          void* dX, int64_t lddx, void* dW, int64_t lddw,
                          int32_t M, int32_t K, int32_t N,
                          const int32_t* keep_idx, int32_t n_keep,
                          int mode, int w_layout, int dtype, int policy,
                          const void* prev_dX, const void* prev_dW,
                          void* workspace, size_t workspace_bytes, int workspace_flags, void* stream);

/* Stand-alone recovery/imputation (Sec. 3.1, "Consistency Constraint": the
 * pruned dimensions are put back, and the three policies): fills every slice of out[rows x cols]
 * that is NOT in keep_idx along `axis` (0: keep_idx indexes rows, 1: columns);
 * kept slices are left as they are.
 *  ZERO: +0.0.  SAME: prev[same position] (prev has out's shape and ld; prev ==
 *  out is allowed and is a no-op).  AVERAGE: mean, in fp32, of the kept slices'
 *  stored values (axis 1: per-row mean over kept columns; axis 0: per-column
 *  mean over kept rows), rounded to the tensor's dtype.
 *  Errors: NULL, SHAPE, INDEX, DTYPE, POLICY, LIMIT, HIP. */
int zr_impute(void* out, int64_t ld, int32_t rows, int32_t cols, int32_t axis,
              const int32_t* keep_idx, int32_t n_keep, int policy, const void* prev,
              int dtype, void* stream);

/* Weight-variation scores (Sec. 3.2 "Priority Pruning"; Algorithm 1):
 *   scores[i] = mean over the slice's elements of |W_t - W_prev|, for every index
 *   i of the pruned axis of W[K x N] (columns for ZR_DROP_N, rows for ZR_DROP_K;
 *   a shard stored [N x K] is passed as that [N x K] matrix with the other mode);
 * incremental update (Sec. 3.2): when prev_keep_idx is given, an index that is
 * NOT in it (it was pruned in the previous epoch) receives prev_scores[i] instead.
 *  W_t, W_prev [K x N] with a common leading dimension ld; scores fp32 [n] out;
 *  prev_keep_idx NULL = plain update (prev_scores ignored).  fp32 sums in a fixed
 *  order, bitwise repeatable for a given workspace size.
 *  workspace: optional device scratch of zr_priority_workspace_bytes(K, N, mode)
 *  bytes (0 for ZR_DROP_K): with it the column sums of ZR_DROP_N are split over
 *  row ranges so that the launch fills the chip (two launches); NULL or too
 *  small = one launch that owns whole columns.  The library never allocates.
 *  Errors: NULL, DTYPE, MODE, SHAPE, INDEX, HIP. */
int zr_priority_scores(const void* W_t, const void* W_prev, int64_t ld, int32_t K, int32_t N, int mode,
                       const float* prev_scores, const int32_t* prev_keep_idx, int32_t n_prev_keep,
                       float* scores, int dtype, void* workspace, size_t workspace_bytes, void* stream);
size_t zr_priority_workspace_bytes(int32_t K, int32_t N, int mode);

/* zr_priority_scores for callers that cannot allocate or pass scratch memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments and results as zr_priority_scores given a workspace of
 * zr_priority_workspace_bytes(K, N, mode) bytes (bit for bit: same row ranges,
 * same summation order), but the per-row-range column sums live in a buffer the
 * library itself holds in device memory: zr_priority_static_scratch_bytes() =
 * 1 MiB per GPU, from the moment the library is loaded on that GPU until the
 * process ends.  The call allocates and frees nothing.  Its first use on a device
 * looks the buffer's address up (once per device; make that first call outside a
 * stream capture).
 *  Limit: zr_priority_workspace_bytes(K, N, mode) <= 1 MiB, else ZR_ERR_LIMIT and
 *  nothing is enqueued (the row-range split needs about 65536 + N floats, so any N
 *  up to about 190000 columns fits; ZR_DROP_K needs no scratch at all).
 *  All calls on one GPU share the buffer, which keeps the last call's contents:
 *  every slot a call reads it has written itself first, so nothing needs
 *  clearing, but two calls that overlap on one GPU (different streams, or
 *  different threads) race on it - order them.
 *  Errors: NULL, DTYPE, MODE, SHAPE, INDEX, LIMIT, HIP. */
int zr_priority_scores_static(const void* W_t, const void* W_prev, int64_t ld, int32_t K, int32_t N, int mode,
                              const float* prev_scores, const int32_t* prev_keep_idx, int32_t n_prev_keep,
                              float* scores, int dtype, void* stream);
size_t zr_priority_static_scratch_bytes(void);

/* Eq. 1: pruning ratio gamma = (T_i - T_avg) / M_i from the task's iteration time,
 * the average iteration time and the task's matrix-multiplication time; 0 when
 * the task is not slower than the average; capped at gamma_max (< 1).  Pure host
 * function; returns -1 on a non-positive M_i or a bad cap. */
double zr_pruning_ratio(double T_i, double T_avg, double M_i, double gamma_max);

/* Differentiated per-layer ratio (Sec. 3.2, Algorithm 1): zr_count_above writes
 * L_uni = #{i : scores[i] > theta} to the DEVICE int32 `count` (one launch, async);
 * zr_layer_ratio (pure host) returns max(1 - L_uni / L, alpha * gamma), or -1 on
 * bad arguments.  theta = N_iter * theta_iter (1e-3 by default in the paper),
 * alpha = 0.8 by default. */
int zr_count_above(const float* scores, int32_t n, float theta, int32_t* count, void* stream);
double zr_layer_ratio(int64_t count_above, int64_t L, double alpha, double gamma);

/* Lightweight migration, one receiver's share (Sec. 4.1 and the renumbering
 * passage of Sec. 4.2).
 * zr_migration_range (pure host): of the straggler's L_mig migrated columns,
 * task r_i computes [*begin, *end): with the straggler at rank r_k among e
 * tasks, r' = (r_i + e - r_k) % e and the range is [m (r'-1), m r' - 1],
 * m = L_mig / (e-1); a remainder is spread one column each over the first
 * receivers; the straggler (r' = 0) gets the empty range.  Errors: NULL, SHAPE.
 * zr_migrated_accumulate: the local reduce that replaces the global one:
 *   out[M x N] += A[M x C] * B           (b_transposed = 0, B is [C x N]: row-parallel forward,
 *                                          A = X_mig[:, range], B = W_mig[range, :])
 *   out[M x N] += A[M x C] * B^T         (b_transposed = 1, B is [N x C]: column-parallel backward,
 *                                          A = dY_mig[:, range], B = W_mig[:, range])
 * A, B, out are DEVICE sub-matrix views (pointer to the first element of the
 * range + leading dimension); the old value of out joins the fp32 accumulator
 * before the single rounding to the output type.  One launch.  16-byte aligned
 * views with leading dimensions that are multiples of 8 run on the fast path.
 * Errors: NULL, DTYPE, SHAPE, HIP. */
int zr_migration_range(int32_t r_i, int32_t r_k, int32_t e, int64_t L_mig, int64_t* begin, int64_t* end);
int zr_migrated_accumulate(const void* A, int64_t lda, const void* B, int64_t ldb, int b_transposed,
                           void* out, int64_t ldo, int32_t M, int32_t N, int32_t C, int dtype, void* stream);

/* Debugging aid: checks on the device that keep_idx[n_keep] is strictly
 * ascending and within [0, n).  SYNCHRONISES `stream`.  `flag` is a caller-owned
 * device int32 used as scratch.  Returns ZR_OK or ZR_ERR_INDEX. */
int zr_validate_keep_idx(const int32_t* keep_idx, int32_t n_keep, int32_t n,
                         int32_t* flag, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ZR_H */

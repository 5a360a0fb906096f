// C ABI of libzr: argument validation and the mapping of the six resized
// products (paper Sec. 3.1) onto the canonical gather-fused GEMM.
#include <cmath>

#include "zr_common.h"

using namespace zr;

namespace {

constexpr size_t kSplitScratchBytes = (size_t)64 << 20;
// the fill kernels of the imputation passes put 32 rows on one workgroup of a grid's second dimension
// (at most 65535 of them)
constexpr int32_t kMaxRows = 65535 * 32;

bool valid_dtype(int dt) { return dt == ZR_F32 || dt == ZR_BF16; }
bool valid_mode(int m) { return m == ZR_DROP_N || m == ZR_DROP_K; }
bool valid_policy(int p) { return p == ZR_IMPUTE_ZERO || p == ZR_IMPUTE_AVERAGE || p == ZR_IMPUTE_SAME; }

int check_common(int32_t M, int32_t K, int32_t N, const int32_t* keep_idx, int32_t n_keep,
                 int mode, int dtype, int policy)
{
    if (!valid_dtype(dtype)) return ZR_ERR_DTYPE;
    if (!valid_mode(mode)) return ZR_ERR_MODE;
    if (!valid_policy(policy)) return ZR_ERR_POLICY;
    if (M < 1 || K < 1 || N < 1) return ZR_ERR_SHAPE;
    if (M > kMaxRows || K > kMaxRows || N > kMaxRows) return ZR_ERR_LIMIT;
    if (!keep_idx) return ZR_ERR_NULL;
    const int32_t n = mode == ZR_DROP_N ? N : K;
    if (n_keep < 1 || n_keep > n) return ZR_ERR_INDEX;
    return ZR_OK;
}

Operand operand(const void* base, int64_t ld, bool c_contig, const int32_t* map_strided,
                const int32_t* map_contig, int n_strided, int n_contig)
{
    Operand o;
    o.base = base; o.ld = ld; o.c_contig = c_contig;
    o.map_strided = map_strided; o.map_contig = map_contig;
    o.n_strided = n_strided; o.n_contig = n_contig;
    o.zero_padded = false;
    return o;
}

// Extracted activation in the caller's workspace: [M x width] bf16, width = n_keep
// rounded up to 64, zero beyond n_keep.  Returns false when the workspace path
// does not apply (then the GEMM loaders gather in flight).
struct Extract {
    bool use;
    int width;
};

int round_up64(int v) { return (v + 63) / 64 * 64; }

Extract plan_extract(const void* src, int64_t ld, int32_t M, int32_t n, int32_t n_keep, int dtype,
                     const void* workspace, size_t workspace_bytes)
{
    Extract e{false, 0};
    if (dtype != ZR_BF16 || !workspace || n_keep == n) return e;
    const int width = round_up64(n_keep);
    if ((size_t)M * (size_t)width * 2 > workspace_bytes) return e;
    if ((uintptr_t)workspace % 16 != 0 || (uintptr_t)src % 4 != 0 || ld % 2 != 0 || n % 2 != 0) return e;
    e.use = true;
    e.width = width;
    return e;
}

// Average imputation through the product's own epilogue: the tail of the caller's
// scratch buffer holds the per-tile sums, ceil(extent / 128) slots of `len` floats
// (extent = kept count along the summed axis, len = length of the other axis).
size_t avg_bytes(int len, int n_keep) { return ((size_t)((n_keep + 127) / 128) * (size_t)len * 4 + 15) & ~(size_t)15; }

// Splits the workspace: returns the sums' address (nullptr: no room, the stand-alone
// second pass is used) and shrinks `bytes` to what is left for the extraction.
float* carve_avg(void* workspace, size_t& bytes, size_t need)
{
    if (!workspace || need == 0 || bytes < need + 16) return nullptr;
    const size_t off = (bytes - need) & ~(size_t)15;
    if ((uintptr_t)workspace % 16 != 0) return nullptr;
    bytes = off;
    return (float*)((char*)workspace + off);
}

// Bytes at the start of the workspace that hold (or may still hold, for a backward call after
// the forward call of the same step) an extracted activation.
size_t extraction_bytes(int32_t M, int32_t n, int32_t n_keep, int dtype, const void* workspace, size_t workspace_bytes)
{
    if (dtype != ZR_BF16 || !workspace || n_keep == n) return 0;
    const size_t need = (size_t)M * (size_t)round_up64(n_keep) * 2;
    return need <= workspace_bytes ? need : 0;
}

// Scratch of a split contraction: what lies between the extracted activation (the first
// `used` bytes) and the end of the buffer (after the Average sums were carved off its tail).
void give_split_scratch(GemmDesc& d, void* workspace, size_t bytes, size_t used)
{
    d.split_scratch = nullptr; d.split_scratch_bytes = 0;
    if (!workspace || (uintptr_t)workspace % 16 != 0) return;
    const size_t off = (used + 15) & ~(size_t)15;
    if (bytes <= off + 16) return;
    d.split_scratch = (char*)workspace + off;
    d.split_scratch_bytes = bytes - off;
}

// One product with Average imputation: zero the sums, multiply (the scatter epilogue
// writes results, +0 and the sums), then mean and fill; or, without room for the
// sums, multiply and run the stand-alone pass that re-reads the kept slices.
int gemm_with_average(GemmDesc& d, float* sums, void* out, int64_t ld, int rows, int cols, int axis,
                      const int32_t* keep_idx, int n_keep, int dtype, hipStream_t s)
{
    int st;
    if (sums) {
        const int len = axis == 1 ? rows : cols;
        const int slots = (n_keep + 127) / 128;
        st = launch_zero_f32(sums, (size_t)slots * (size_t)len, s);
        if (st != ZR_OK) return st;
        d.avg_partial = sums; d.avg_len = len;
        st = launch_gemm(d, s);
        d.avg_partial = nullptr;
        if (st != ZR_OK) return st;
        return launch_mean_fill(out, ld, rows, cols, axis, keep_idx, n_keep, sums, slots, dtype, s);
    }
    st = launch_gemm(d, s);
    if (st != ZR_OK) return st;
    return launch_impute(out, ld, rows, cols, axis, keep_idx, n_keep, ZR_IMPUTE_AVERAGE, nullptr, dtype, s);
}

}  // namespace

extern "C" {

size_t zr_workspace_bytes(int32_t M, int32_t K, int32_t N, int32_t n_keep, int mode, int dtype)
{
    (void)mode;
    if (M < 1 || K < 1 || N < 1 || n_keep < 1) return 0;
    // extracted activation columns [M x width] (bf16 only), then the per-tile sums of Average imputation
    const size_t act = dtype == ZR_BF16 ? (size_t)M * (size_t)round_up64(n_keep) * 2 : 0;
    // + room for the slices of a split contraction (bf16 products with too few tiles for the chip)
    const size_t split = dtype == ZR_BF16 ? kSplitScratchBytes : 0;
    return act + 16 + split + avg_bytes(std::max(M, std::max(K, N)), n_keep) + 16;
}

const char* zr_status_string(int status)
{
    switch (status) {
        case ZR_OK: return "ok";
        case ZR_ERR_NULL: return "a required pointer is NULL";
        case ZR_ERR_SHAPE: return "bad shape or leading dimension";
        case ZR_ERR_RATIO: return "ratio outside [0,1) or no index kept";
        case ZR_ERR_INDEX: return "bad kept count or kept-index list";
        case ZR_ERR_DTYPE: return "unknown dtype";
        case ZR_ERR_MODE: return "unknown mode";
        case ZR_ERR_POLICY: return "unknown policy or missing previous tensor";
        case ZR_ERR_LIMIT: return "size beyond the supported limit";
        case ZR_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

void zr_debug_record_kernel_names(int on) { g_debug.record_names = on != 0; }

const char* zr_debug_last_kernel(void) { return g_debug.last_kernel; }

int zr_debug_time_next_product(void* start_event, void* stop_event)
{
    if (!start_event || !stop_event) return ZR_ERR_NULL;
    g_debug.start = (hipEvent_t)start_event;
    g_debug.stop = (hipEvent_t)stop_event;
    g_debug.armed_once = true;
    return ZR_OK;
}

int zr_debug_mfma_rate(int32_t blocks, int32_t iters, float* sink, double* flops, void* stream)
{
    if (!sink) return ZR_ERR_NULL;
    if (blocks < 1 || iters < 1 || blocks > (1 << 20)) return ZR_ERR_SHAPE;
    if (flops) *flops = mfma_rate_flops(blocks, iters);
    return launch_mfma_rate(blocks, iters, sink, (hipStream_t)stream);
}

int zr_extract_kept_columns(const void* in, int64_t ld, int32_t rows, int32_t n,
                            const int32_t* keep_idx, int32_t n_keep,
                            void* out, int64_t ldo, int dtype, void* stream)
{
    if (!in || !keep_idx || !out) return ZR_ERR_NULL;
    if (dtype != ZR_BF16) return ZR_ERR_DTYPE;
    if (rows < 1 || n < 1 || ld < n) return ZR_ERR_SHAPE;
    if (n_keep < 1 || n_keep > n) return ZR_ERR_INDEX;
    const int width = round_up64(n_keep);
    if (ldo < width || ldo % 2 != 0 || ld % 2 != 0 || n % 2 != 0) return ZR_ERR_SHAPE;
    if ((uintptr_t)in % 4 != 0 || (uintptr_t)out % 4 != 0) return ZR_ERR_SHAPE;
    return launch_compact_cols(in, ld, rows, n, keep_idx, n_keep, out, ldo, width, (hipStream_t)stream);
}

int64_t zr_keep_count(int64_t n, double ratio)
{
    if (n < 0 || !(ratio >= 0.0) || !(ratio < 1.0)) return -1;
    // floor((1 - ratio) * n + 0.5) with every operation rounded to double
    // (no fused multiply-add: the product is stored before the addition)
    volatile double kept = (1.0 - ratio) * (double)n;
    volatile double shifted = kept + 0.5;
    return (int64_t)std::floor(shifted);
}

int zr_resize_select(const float* scores, int32_t n, int32_t batch, double ratio,
                     int32_t* keep_idx, int32_t* drop_idx, int64_t ld_idx, void* stream)
{
    if (!scores || !keep_idx) return ZR_ERR_NULL;
    if (n < 1 || batch < 1) return ZR_ERR_SHAPE;
    if (n > (1 << 24)) return ZR_ERR_LIMIT;
    const int64_t n_keep = zr_keep_count(n, ratio);
    if (n_keep < 1) return ZR_ERR_RATIO;
    if (ld_idx < n_keep || (drop_idx && ld_idx < n - n_keep)) return ZR_ERR_SHAPE;
    return launch_select(scores, n, batch, (int)n_keep, keep_idx, drop_idx, ld_idx, (hipStream_t)stream);
}

size_t zr_select_workspace_bytes(int32_t n)
{
    if (n < 1) return 0;
    return n >= select_wide_min_n() ? select_wide_workspace_bytes() : 0;
}

int zr_resize_select_ws(const float* scores, int32_t n, double ratio, int32_t* keep_idx, int32_t* drop_idx,
                        void* workspace, size_t workspace_bytes, void* stream)
{
    if (!scores || !keep_idx) return ZR_ERR_NULL;
    if (n < 1) return ZR_ERR_SHAPE;
    if (n > (1 << 24)) return ZR_ERR_LIMIT;
    const int64_t n_keep = zr_keep_count(n, ratio);
    if (n_keep < 1) return ZR_ERR_RATIO;
    const bool wide = n >= select_wide_min_n() && workspace && (uintptr_t)workspace % 4 == 0 &&
                      workspace_bytes >= select_wide_workspace_bytes();
    if (!wide) return launch_select(scores, n, 1, (int)n_keep, keep_idx, drop_idx, n, (hipStream_t)stream);
    return launch_select_wide(scores, n, (int)n_keep, keep_idx, drop_idx, workspace, (hipStream_t)stream);
}

int zr_resize_select_multi(int32_t count, const float* const* scores, const int32_t* n, const double* ratio,
                           int32_t* const* keep_idx, int32_t* const* drop_idx, void* stream)
{
    if (!scores || !n || !ratio || !keep_idx) return ZR_ERR_NULL;
    if (count < 1) return ZR_ERR_SHAPE;
    if (count > ZR_SELECT_MULTI_MAX) return ZR_ERR_LIMIT;
    SelectMulti m;
    for (int b = 0; b < count; ++b) {
        if (!scores[b] || !keep_idx[b]) return ZR_ERR_NULL;
        if (n[b] < 1) return ZR_ERR_SHAPE;
        if (n[b] > (1 << 24)) return ZR_ERR_LIMIT;
        const int64_t n_keep = zr_keep_count(n[b], ratio[b]);
        if (n_keep < 1) return ZR_ERR_RATIO;
        m.scores[b] = scores[b]; m.keep[b] = keep_idx[b]; m.drop[b] = drop_idx ? drop_idx[b] : nullptr;
        m.n[b] = n[b]; m.n_keep[b] = (int)n_keep;
    }
    for (int b = count; b < ZR_SELECT_MULTI_MAX; ++b) {
        m.scores[b] = nullptr; m.keep[b] = nullptr; m.drop[b] = nullptr; m.n[b] = 0; m.n_keep[b] = 0;
    }
    return launch_select_multi(m, count, (hipStream_t)stream);
}

// The weight operand B(j,c) of the three products for both storage layouts of the
// shard: KN = W[K x N] row-major, NK = W^T stored as [N x K] row-major (the
// [out, in] layout).  Whichever axis the kept list indexes, one of the layouts
// makes it the ROW axis of the stored matrix, so that the list only selects
// contiguous rows and the weight is neither gathered element-wise nor copied.
static Operand weight_fwd(const void* W, int64_t ldw, int K, int N, int mode, int layout, const int32_t* S)
{
    // forward: B(j,c) = W[c,j], c over K (DROP_K: c -> S[c]; DROP_N: j -> S[j])
    if (layout == ZR_W_KN)
        return mode == ZR_DROP_K ? operand(W, ldw, false, S, nullptr, K, N) : operand(W, ldw, false, nullptr, S, K, N);
    return mode == ZR_DROP_K ? operand(W, ldw, true, nullptr, S, N, K) : operand(W, ldw, true, S, nullptr, N, K);
}

static Operand weight_dx(const void* W, int64_t ldw, int K, int N, int mode, int layout, const int32_t* S)
{
    // dX: B(j,c) = W[j,c], j over K, c over N (DROP_K: j -> S[j]; DROP_N: c -> S[c])
    if (layout == ZR_W_KN)
        return mode == ZR_DROP_K ? operand(W, ldw, true, S, nullptr, K, N) : operand(W, ldw, true, nullptr, S, K, N);
    return mode == ZR_DROP_K ? operand(W, ldw, false, nullptr, S, N, K) : operand(W, ldw, false, S, nullptr, N, K);
}

int zr_resized_linear_fwd(const void* X, int64_t ldx, const void* W, int64_t ldw,
                          void* Y, int64_t ldy, int32_t M, int32_t K, int32_t N,
                          const int32_t* keep_idx, int32_t n_keep,
                          int mode, int w_layout, int dtype, int policy, const void* prev_Y,
                          void* workspace, size_t workspace_bytes, void* stream)
{
    if (!X || !W || !Y) return ZR_ERR_NULL;
    int st = check_common(M, K, N, keep_idx, n_keep, mode, dtype, policy);
    if (st != ZR_OK) return st;
    if (w_layout != ZR_W_KN && w_layout != ZR_W_NK) return ZR_ERR_MODE;
    if (ldx < K || ldw < (w_layout == ZR_W_KN ? N : K) || ldy < N) return ZR_ERR_SHAPE;
    const bool full = n_keep == (mode == ZR_DROP_N ? N : K);   // ascending + unique + full count = identity
    const bool needs_prev = mode == ZR_DROP_N && policy == ZR_IMPUTE_SAME && !full;
    if (needs_prev && !prev_Y) return ZR_ERR_POLICY;
    hipStream_t s = (hipStream_t)stream;
    const int32_t* S = full ? nullptr : keep_idx;
    const bool average = mode == ZR_DROP_N && policy == ZR_IMPUTE_AVERAGE && !full;
    float* sums = average ? carve_avg(workspace, workspace_bytes, avg_bytes(M, n_keep)) : nullptr;

    GemmDesc d;
    d.dtype = dtype;
    d.out = Y; d.ldo = ldy; d.keep_idx = S; d.I = M;
    d.B = weight_fwd(W, ldw, K, N, mode, w_layout, S);
    if (mode == ZR_DROP_K) {
        // Y[m,j] = sum_{c<n'} X[m,S[c]] * W[S[c],j]
        const Extract ex = plan_extract(X, ldx, M, K, n_keep, dtype, workspace, workspace_bytes);
        if (ex.use) {
            st = launch_compact_cols(X, ldx, M, K, keep_idx, n_keep, workspace, ex.width, ex.width, s);
            if (st != ZR_OK) return st;
            d.A = operand(workspace, ex.width, true, nullptr, nullptr, M, ex.width);
            d.A.zero_padded = true;
        } else {
            d.A = operand(X, ldx, true, nullptr, S, M, K);
        }
        d.J = N; d.C = n_keep; d.epilogue = EPI_PLAIN; d.out_full = N;
        give_split_scratch(d, workspace, workspace_bytes, extraction_bytes(M, K, n_keep, dtype, workspace, workspace_bytes));
        return launch_gemm(d, s);
    }
    // Y[m,S[j]] = sum_k X[m,k] * W[k,S[j]], dropped columns imputed
    d.A = operand(X, ldx, true, nullptr, nullptr, M, K);
    d.J = n_keep; d.C = K; d.epilogue = full ? EPI_PLAIN : EPI_COL_SCATTER; d.out_full = N;
    if (needs_prev) d.prev = prev_Y;            // Same: copied by the scatter epilogue itself
    give_split_scratch(d, workspace, workspace_bytes, 0);
    if (average) return gemm_with_average(d, sums, Y, ldy, M, N, 1, keep_idx, n_keep, dtype, s);
    return launch_gemm(d, s);
}

int zr_resized_linear_bwd(const void* X, int64_t ldx, const void* W, int64_t ldw,
                          const void* dY, int64_t lddy,
                          void* dX, int64_t lddx, void* dW, int64_t lddw,
                          int32_t M, int32_t K, int32_t N,
                          const int32_t* keep_idx, int32_t n_keep,
                          int mode, int w_layout, int dtype, int policy,
                          const void* prev_dX, const void* prev_dW,
                          void* workspace, size_t workspace_bytes, int workspace_flags, void* stream)
{
    if (!dY || (!dX && !dW)) return ZR_ERR_NULL;
    if ((dX && !W) || (dW && !X)) return ZR_ERR_NULL;
    int st = check_common(M, K, N, keep_idx, n_keep, mode, dtype, policy);
    if (st != ZR_OK) return st;
    if (w_layout != ZR_W_KN && w_layout != ZR_W_NK) return ZR_ERR_MODE;
    const bool kn = w_layout == ZR_W_KN;
    if (lddy < N) return ZR_ERR_SHAPE;
    if (dX && (ldw < (kn ? N : K) || lddx < K)) return ZR_ERR_SHAPE;
    if (dW && (ldx < K || lddw < (kn ? N : K))) return ZR_ERR_SHAPE;
    const bool full = n_keep == (mode == ZR_DROP_N ? N : K);
    if (policy == ZR_IMPUTE_SAME && !full) {
        if (dW && !prev_dW) return ZR_ERR_POLICY;
        if (dX && mode == ZR_DROP_K && !prev_dX) return ZR_ERR_POLICY;
    }
    hipStream_t s = (hipStream_t)stream;
    const int32_t* S = full ? nullptr : keep_idx;
    const bool same = !full && policy == ZR_IMPUTE_SAME;       // fused into the scatter epilogues
    const bool post = !full && policy == ZR_IMPUTE_AVERAGE;    // sums in the epilogue, then mean and fill
    float* sums = nullptr;
    if (post) {
        size_t need = 0;
        if (dX && mode == ZR_DROP_K) need = avg_bytes(M, n_keep);
        if (dW) need = std::max(need, avg_bytes(mode == ZR_DROP_K ? N : K, n_keep));
        sums = carve_avg(workspace, workspace_bytes, need);
    }

    // one extraction serves both products: X[:,S] (DROP_K, used by dW) or dY[:,S] (DROP_N)
    Extract ex{false, 0};
    if (mode == ZR_DROP_K) {
        if (dW) ex = plan_extract(X, ldx, M, K, n_keep, dtype, workspace, workspace_bytes);
        // the forward call of this layer left X[:,S] at the same place (same plan, same sizes)
        const bool reuse = (workspace_flags & ZR_WS_HOLDS_FORWARD) != 0;
        if (ex.use && !reuse)
            st = launch_compact_cols(X, ldx, M, K, keep_idx, n_keep, workspace, ex.width, ex.width, s);
    } else {
        ex = plan_extract(dY, lddy, M, N, n_keep, dtype, workspace, workspace_bytes);
        if (ex.use) st = launch_compact_cols(dY, lddy, M, N, keep_idx, n_keep, workspace, ex.width, ex.width, s);
    }
    if (st != ZR_OK) return st;

    GemmDesc d;
    d.dtype = dtype;
    d.keep_idx = S;
    // (in DROP_K the start of the buffer may hold the forward call's X[:,S] even when this call
    // extracts nothing itself)
    give_split_scratch(d, workspace, workspace_bytes,
                       extraction_bytes(M, mode == ZR_DROP_K ? K : N, n_keep, dtype, workspace, workspace_bytes));
    if (dX) {
        d.out = dX; d.ldo = lddx; d.I = M;
        d.B = weight_dx(W, ldw, K, N, mode, w_layout, S);
        if (mode == ZR_DROP_K) {
            // dX[m,S[j]] = sum_n dY[m,n] * W[S[j],n], dropped columns imputed
            d.A = operand(dY, lddy, true, nullptr, nullptr, M, N);
            d.J = n_keep; d.C = N; d.epilogue = full ? EPI_PLAIN : EPI_COL_SCATTER; d.out_full = K;
            if (same) d.prev = prev_dX;
        } else {
            // dX[m,k] = sum_{c<n'} dY[m,S[c]] * W[k,S[c]]
            if (ex.use) {
                d.A = operand(workspace, ex.width, true, nullptr, nullptr, M, ex.width);
                d.A.zero_padded = true;
            } else {
                d.A = operand(dY, lddy, true, nullptr, S, M, N);
            }
            d.J = K; d.C = n_keep; d.epilogue = EPI_PLAIN; d.out_full = K;
        }
        if (post && mode == ZR_DROP_K) st = gemm_with_average(d, sums, dX, lddx, M, K, 1, keep_idx, n_keep, dtype, s);
        else st = launch_gemm(d, s);
        if (st != ZR_OK) return st;
    }
    if (dW) {
        // dW has the layout of W.  KN: D[i=k, j=n]; NK: D[i=n, j=k]; contraction over the tokens.
        d.out = dW; d.ldo = lddw; d.C = M;
        d.prev = same ? prev_dW : nullptr;
        const Operand xs = (mode == ZR_DROP_K)
            ? (ex.use ? operand(workspace, ex.width, false, nullptr, nullptr, M, ex.width)
                      : operand(X, ldx, false, nullptr, S, M, K))
            : operand(X, ldx, false, nullptr, nullptr, M, K);
        const Operand dys = (mode == ZR_DROP_N)
            ? (ex.use ? operand(workspace, ex.width, false, nullptr, nullptr, M, ex.width)
                      : operand(dY, lddy, false, nullptr, S, M, N))
            : operand(dY, lddy, false, nullptr, nullptr, M, N);
        const int ik = mode == ZR_DROP_K ? n_keep : K;       // extent of the K index of D
        const int in = mode == ZR_DROP_N ? n_keep : N;       // extent of the N index of D
        // the kept list indexes rows of the stored dW in (KN, DROP_K) and (NK, DROP_N), columns otherwise
        const bool rows_pruned = kn == (mode == ZR_DROP_K);
        if (kn) { d.A = xs; d.B = dys; d.I = ik; d.J = in; }
        else    { d.A = dys; d.B = xs; d.I = in; d.J = ik; }
        d.epilogue = full ? EPI_PLAIN : (rows_pruned ? EPI_ROW_SCATTER : EPI_COL_SCATTER);
        d.out_full = mode == ZR_DROP_K ? K : N;
        if (post) st = gemm_with_average(d, sums, dW, lddw, kn ? K : N, kn ? N : K, rows_pruned ? 0 : 1, keep_idx,
                                         n_keep, dtype, s);
        else st = launch_gemm(d, s);
        if (st != ZR_OK) return st;
    }
    return ZR_OK;
}

int zr_priority_scores(const void* W_t, const void* W_prev, int64_t ld, int32_t K, int32_t N, int mode,
                       const float* prev_scores, const int32_t* prev_keep_idx, int32_t n_prev_keep,
                       float* scores, int dtype, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!W_t || !W_prev || !scores) return ZR_ERR_NULL;
    if (!valid_dtype(dtype)) return ZR_ERR_DTYPE;
    if (!valid_mode(mode)) return ZR_ERR_MODE;
    if (K < 1 || N < 1 || ld < N) return ZR_ERR_SHAPE;
    if (prev_keep_idx) {
        if (!prev_scores) return ZR_ERR_NULL;
        const int32_t n = mode == ZR_DROP_N ? N : K;
        if (n_prev_keep < 1 || n_prev_keep > n) return ZR_ERR_INDEX;
    }
    return launch_priority_scores(W_t, W_prev, ld, K, N, mode, prev_scores, prev_keep_idx, n_prev_keep, scores,
                                  dtype, workspace, workspace_bytes, (hipStream_t)stream);
}

int zr_priority_scores_static(const void* W_t, const void* W_prev, int64_t ld, int32_t K, int32_t N, int mode,
                              const float* prev_scores, const int32_t* prev_keep_idx, int32_t n_prev_keep,
                              float* scores, int dtype, void* stream)
{
    if (!W_t || !W_prev || !scores) return ZR_ERR_NULL;
    if (!valid_dtype(dtype)) return ZR_ERR_DTYPE;
    if (!valid_mode(mode)) return ZR_ERR_MODE;
    if (K < 1 || N < 1 || ld < N) return ZR_ERR_SHAPE;
    if (prev_keep_idx) {
        if (!prev_scores) return ZR_ERR_NULL;
        const int32_t n = mode == ZR_DROP_N ? N : K;
        if (n_prev_keep < 1 || n_prev_keep > n) return ZR_ERR_INDEX;
    }
    return launch_priority_scores_static(W_t, W_prev, ld, K, N, mode, prev_scores, prev_keep_idx, n_prev_keep,
                                         scores, dtype, (hipStream_t)stream);
}

size_t zr_priority_static_scratch_bytes(void) { return priority_static_scratch_bytes(); }

size_t zr_priority_workspace_bytes(int32_t K, int32_t N, int mode)
{
    if (K < 1 || N < 1 || !valid_mode(mode)) return 0;
    return priority_workspace_bytes(K, N, mode);
}

double zr_pruning_ratio(double T_i, double T_avg, double M_i, double gamma_max)
{
    if (!(M_i > 0.0) || !(gamma_max >= 0.0) || !(gamma_max < 1.0)) return -1.0;
    const double g = (T_i - T_avg) / M_i;
    if (!(g > 0.0)) return 0.0;          // not slower than the average (or NaN): prune nothing
    return g < gamma_max ? g : gamma_max;
}

int zr_count_above(const float* scores, int32_t n, float theta, int32_t* count, void* stream)
{
    if (!scores || !count) return ZR_ERR_NULL;
    if (n < 1) return ZR_ERR_SHAPE;
    return launch_count_above(scores, n, theta, count, (hipStream_t)stream);
}

double zr_layer_ratio(int64_t count_above, int64_t L, double alpha, double gamma)
{
    if (L < 1 || count_above < 0 || count_above > L) return -1.0;
    const double gk = 1.0 - (double)count_above / (double)L;
    const double floor_ = alpha * gamma;
    return gk > floor_ ? gk : floor_;
}

int zr_migration_range(int32_t r_i, int32_t r_k, int32_t e, int64_t L_mig, int64_t* begin, int64_t* end)
{
    if (!begin || !end) return ZR_ERR_NULL;
    if (e < 2 || r_i < 0 || r_k < 0 || L_mig < 0) return ZR_ERR_SHAPE;
    const int64_t r_new = ((int64_t)r_i + e - r_k) % e;
    if (r_new == 0) { *begin = 0; *end = 0; return ZR_OK; }      // the straggler itself
    const int64_t m = L_mig / (e - 1), rem = L_mig % (e - 1);
    const int64_t b = m * (r_new - 1) + std::min<int64_t>(r_new - 1, rem);
    *begin = b;
    *end = b + m + (r_new - 1 < rem ? 1 : 0);
    return ZR_OK;
}

int zr_migrated_accumulate(const void* A, int64_t lda, const void* B, int64_t ldb, int b_transposed,
                           void* out, int64_t ldo, int32_t M, int32_t N, int32_t C, int dtype, void* stream)
{
    if (!A || !B || !out) return ZR_ERR_NULL;
    if (!valid_dtype(dtype)) return ZR_ERR_DTYPE;
    if (M < 1 || N < 1 || C < 1) return ZR_ERR_SHAPE;
    if (lda < C || ldo < N || ldb < (b_transposed ? C : N)) return ZR_ERR_SHAPE;
    GemmDesc d;
    d.dtype = dtype;
    d.out = out; d.ldo = ldo; d.keep_idx = nullptr; d.out_full = N;
    d.I = M; d.J = N; d.C = C; d.epilogue = EPI_PLAIN;
    d.accumulate = true;
    d.A = operand(A, lda, true, nullptr, nullptr, M, C);
    // out[m,n] += sum_c A[m,c] * B[c,n]   or   sum_c A[m,c] * B[n,c]
    d.B = b_transposed ? operand(B, ldb, true, nullptr, nullptr, N, C)
                       : operand(B, ldb, false, nullptr, nullptr, C, N);
    return launch_gemm(d, (hipStream_t)stream);
}

int zr_impute(void* out, int64_t ld, int32_t rows, int32_t cols, int32_t axis,
              const int32_t* keep_idx, int32_t n_keep, int policy, const void* prev,
              int dtype, void* stream)
{
    if (!out || !keep_idx) return ZR_ERR_NULL;
    if (!valid_dtype(dtype)) return ZR_ERR_DTYPE;
    if (!valid_policy(policy)) return ZR_ERR_POLICY;
    if (rows < 1 || cols < 1 || ld < cols || (axis != 0 && axis != 1)) return ZR_ERR_SHAPE;
    const int32_t n = axis == 0 ? rows : cols;
    if (n_keep < 1 || n_keep > n) return ZR_ERR_INDEX;
    if (policy == ZR_IMPUTE_SAME && n_keep < n && !prev) return ZR_ERR_POLICY;
    if (rows > kMaxRows) return ZR_ERR_LIMIT;
    return launch_impute(out, ld, rows, cols, axis, keep_idx, n_keep, policy, prev, dtype,
                         (hipStream_t)stream);
}

int zr_validate_keep_idx(const int32_t* keep_idx, int32_t n_keep, int32_t n,
                         int32_t* flag, void* stream)
{
    if (!keep_idx || !flag) return ZR_ERR_NULL;
    if (n < 1 || n_keep < 1 || n_keep > n) return ZR_ERR_INDEX;
    return launch_validate(keep_idx, n_keep, n, flag, (hipStream_t)stream);
}

}  // extern "C"

// Stand-ins for the kernel launchers of libzr, for the host-only sanitizer build of the
// C ABI's argument validation and product mapping (zr_api.hip).  Nothing here touches a
// GPU: every launcher checks the description it was handed for the invariants the real
// kernels rely on and counts the call.
#include <cstdio>
#include <cstdlib>

#include "zr_common.h"

namespace zr {

thread_local DebugState g_debug;
int g_launches = 0;
const char* g_ws_begin = nullptr;      // the workspace of the call under test (set by the driver)
const char* g_ws_end = nullptr;

static void require(bool ok, const char* what)
{
    if (!ok) { fprintf(stderr, "stub invariant violated: %s\n", what); abort(); }
}

static void check_operand(const Operand& o)
{
    require(o.base != nullptr, "operand base");
    require(o.ld >= 1 && o.n_strided >= 1 && o.n_contig >= 1, "operand extents");
    require(!(o.map_strided && o.map_contig), "at most one list per operand");
}

int launch_gemm(const GemmDesc& d, hipStream_t)
{
    ++g_launches;
    check_operand(d.A); check_operand(d.B);
    require(d.I >= 1 && d.J >= 1 && d.C >= 1 && d.out && d.ldo >= 1, "product extents");
    require(d.epilogue == EPI_PLAIN || d.keep_idx != nullptr, "scatter epilogue without a list");
    require(d.epilogue == EPI_PLAIN || d.out_full >= (d.epilogue == EPI_COL_SCATTER ? d.J : d.I), "scatter range");
    require(!d.accumulate || d.epilogue == EPI_PLAIN, "accumulate only with the plain epilogue");
    if (d.split_scratch) {
        const char* p = (const char*)d.split_scratch;
        require((uintptr_t)p % 16 == 0, "split scratch alignment");
        require(g_ws_begin && p >= g_ws_begin && p + d.split_scratch_bytes <= g_ws_end, "split scratch outside the workspace");
        // an operand that lives in the workspace (an extracted activation) is never overlapped
        for (const Operand* o : {&d.A, &d.B}) {
            const char* b = (const char*)o->base;
            if (b >= g_ws_begin && b < g_ws_end)
                require(p >= b + (size_t)o->n_strided * (size_t)o->ld * 2, "split scratch overlaps an extracted operand");
        }
    }
    if (d.avg_partial) {
        const char* p = (const char*)d.avg_partial;
        require(g_ws_begin && p >= g_ws_begin && p < g_ws_end, "average sums outside the workspace");
        require(!d.split_scratch || (const char*)d.split_scratch + d.split_scratch_bytes <= p, "split scratch runs into the sums");
    }
    return ZR_OK;
}
int launch_gemm_fast(const GemmDesc&, hipStream_t) { return -1; }
int launch_select(const float* s, int n, int batch, int n_keep, int32_t* k, int32_t*, int64_t ld, hipStream_t)
{
    ++g_launches;
    require(s && k && n >= 1 && batch >= 1 && n_keep >= 1 && n_keep <= n && ld >= n_keep, "select arguments");
    return ZR_OK;
}
size_t select_wide_workspace_bytes() { return (1032 + 4 * 4096) * 4; }
int select_wide_min_n() { return 131072; }
int launch_select_wide(const float* s, int n, int n_keep, int32_t* k, int32_t*, void* ws, hipStream_t)
{
    ++g_launches;
    require(s && k && ws && n >= select_wide_min_n() && n_keep >= 1 && n_keep <= n, "wide select arguments");
    return ZR_OK;
}
int launch_select_multi(const SelectMulti& m, int count, hipStream_t)
{
    ++g_launches;
    require(count >= 1 && count <= ZR_SELECT_MULTI_MAX, "select_multi count");
    for (int b = 0; b < count; ++b) require(m.scores[b] && m.keep[b] && m.n_keep[b] >= 1 && m.n_keep[b] <= m.n[b], "select_multi entry");
    return ZR_OK;
}
int launch_impute(void* out, int64_t ld, int rows, int cols, int axis, const int32_t* keep, int n_keep, int policy,
                  const void* prev, int, hipStream_t)
{
    ++g_launches;
    require(out && keep && ld >= cols && rows >= 1 && (axis == 0 || axis == 1) && n_keep >= 1, "impute arguments");
    require(policy != ZR_IMPUTE_SAME || prev || n_keep == (axis ? cols : rows), "same without previous tensor");
    return ZR_OK;
}
int launch_zero_f32(float* p, size_t count, hipStream_t) { ++g_launches; require(p && count > 0, "zero fill"); return ZR_OK; }
int launch_mean_fill(void* out, int64_t, int, int, int, const int32_t* keep, int, float* partial, int slots, int, hipStream_t)
{
    ++g_launches;
    require(out && keep && partial && slots >= 1, "mean fill");
    return ZR_OK;
}
int launch_compact_cols(const void* in, int64_t ld, int rows, int n, const int32_t* keep, int n_keep, void* out, int64_t ldo,
                        int width, hipStream_t)
{
    ++g_launches;
    require(in && keep && out && rows >= 1 && n_keep >= 1 && n_keep <= n && ld >= n && width % 64 == 0 && width >= n_keep && ldo >= width,
            "extraction arguments");
    return ZR_OK;
}
int launch_priority_scores(const void* a, const void* b, int64_t ld, int K, int N, int, const float*, const int32_t*, int, float* s,
                           int, void*, size_t, hipStream_t)
{
    ++g_launches;
    require(a && b && s && K >= 1 && N >= 1 && ld >= N, "priority arguments");
    return ZR_OK;
}
int launch_priority_scores_static(const void* a, const void* b, int64_t ld, int K, int N, int mode, const float* ps, const int32_t* pk,
                                  int npk, float* s, int dtype, hipStream_t st)
{
    if (priority_workspace_bytes(K, N, mode) > priority_static_scratch_bytes()) return ZR_ERR_LIMIT;
    return launch_priority_scores(a, b, ld, K, N, mode, ps, pk, npk, s, dtype, nullptr, 0, st);
}
size_t priority_workspace_bytes(int K, int N, int mode) { return mode == ZR_DROP_N ? (size_t)(65536 + N) * 4 + (size_t)(K > 0) : 0; }
size_t priority_static_scratch_bytes() { return (size_t)1 << 20; }
int launch_count_above(const float* s, int n, float, int32_t* c, hipStream_t) { ++g_launches; require(s && c && n >= 1, "count"); return ZR_OK; }
int launch_mfma_rate(int blocks, int iters, float* sink, hipStream_t) { ++g_launches; require(blocks >= 1 && iters >= 1 && sink, "probe"); return ZR_OK; }
double mfma_rate_flops(int blocks, int iters) { return 2.0 * blocks * iters; }
int launch_validate(const int32_t* k, int n_keep, int n, int32_t* flag, hipStream_t) { ++g_launches; require(k && flag && n_keep <= n, "validate"); return ZR_OK; }

}  // namespace zr

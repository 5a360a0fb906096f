// Host-only driver of the C ABI (zr.h) for the sanitizer build: every entry point with bad
// and good arguments, return codes checked.  Pointers that stand for device memory are never
// dereferenced by the host code under test; the workspace is a real host buffer so that the
// stubs can check where the calls place their scratch areas.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "zr.h"
#include "zr_debug.h"

namespace zr { extern int g_launches; extern const char* g_ws_begin; extern const char* g_ws_end; }

static int failures = 0;
#define EXPECT(cond) do { if (!(cond)) { fprintf(stderr, "FAILED line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

int main()
{
    alignas(16) static char dev[256];             // any non-null "device" address
    void* P = dev;
    int32_t* KI = (int32_t*)dev;
    float* SC = (float*)dev;

    // ---- pure host functions
    EXPECT(zr_keep_count(10, 0.25) == 8 && zr_keep_count(3072, 0.5) == 1536 && zr_keep_count(0, 0.0) == 0);
    EXPECT(zr_keep_count(-1, 0.0) == -1 && zr_keep_count(8, 1.0) == -1 && zr_keep_count(8, -0.1) == -1 && zr_keep_count(8, NAN) == -1);
    for (int st = -1; st <= 12; ++st) EXPECT(zr_status_string(st) != nullptr && strlen(zr_status_string(st)) > 0);
    EXPECT(zr_pruning_ratio(12, 10, 8, 0.9) == 0.25 && zr_pruning_ratio(9, 10, 8, 0.9) == 0.0 && zr_pruning_ratio(1, 1, 0, 0.9) == -1.0);
    EXPECT(zr_pruning_ratio(NAN, 1, 1, 0.5) == 0.0 && zr_pruning_ratio(5, 1, 1, 1.0) == -1.0);
    EXPECT(zr_layer_ratio(10, 100, 0.8, 0.5) == 0.9 && zr_layer_ratio(100, 100, 0.8, 0.5) == 0.4 && zr_layer_ratio(101, 100, 0.8, 0.5) == -1.0);
    for (int e = 2; e <= 9; ++e)
        for (int rk = 0; rk < e; ++rk)
            for (int64_t L = 0; L <= 40; ++L) {
                int64_t covered = 0, prev_end = 0;
                for (int rp = 1; rp < e; ++rp) {            // receivers in renumbered order tile [0, L)
                    int64_t b = -1, en = -1;
                    EXPECT(zr_migration_range((rk + rp) % e, rk, e, L, &b, &en) == ZR_OK);
                    EXPECT(b == prev_end && en >= b);
                    prev_end = en; covered += en - b;
                }
                EXPECT(covered == L);
                int64_t b = 7, en = 7;
                EXPECT(zr_migration_range(rk, rk, e, L, &b, &en) == ZR_OK && b == 0 && en == 0);
            }
    { int64_t b, en; EXPECT(zr_migration_range(0, 0, 1, 4, &b, &en) == ZR_ERR_SHAPE && zr_migration_range(0, 0, 2, 4, nullptr, &en) == ZR_ERR_NULL); }
    EXPECT(zr_workspace_bytes(0, 8, 8, 4, 0, ZR_BF16) == 0 && zr_workspace_bytes(8, 8, 8, 4, 0, ZR_BF16) > 0);
    EXPECT(zr_priority_workspace_bytes(0, 8, 0) == 0 && zr_priority_workspace_bytes(8, 8, 7) == 0);
    EXPECT(zr_priority_static_scratch_bytes() == (size_t)1 << 20);

    // ---- selection
    EXPECT(zr_resize_select(nullptr, 8, 1, 0.25, KI, KI, 8, nullptr) == ZR_ERR_NULL);
    EXPECT(zr_resize_select(SC, 0, 1, 0.25, KI, KI, 8, nullptr) == ZR_ERR_SHAPE);
    EXPECT(zr_resize_select(SC, 8, 0, 0.25, KI, KI, 8, nullptr) == ZR_ERR_SHAPE);
    EXPECT(zr_resize_select(SC, (1 << 24) + 1, 1, 0.25, KI, KI, 1 << 25, nullptr) == ZR_ERR_LIMIT);
    EXPECT(zr_resize_select(SC, 8, 1, 1.0, KI, KI, 8, nullptr) == ZR_ERR_RATIO);
    EXPECT(zr_resize_select(SC, 8, 1, 0.99, KI, KI, 8, nullptr) == ZR_ERR_RATIO);        // keeps nothing
    EXPECT(zr_resize_select(SC, 8, 1, 0.25, KI, KI, 5, nullptr) == ZR_ERR_SHAPE);        // ld < n'
    EXPECT(zr_resize_select(SC, 8, 1, 0.75, KI, KI, 5, nullptr) == ZR_ERR_SHAPE);        // ld < n - n'
    EXPECT(zr_resize_select(SC, 8, 3, 0.25, KI, nullptr, 6, nullptr) == ZR_OK);
    // the many-workgroup form: same argument checks; a short vector, a missing or a small buffer take the single workgroup
    EXPECT(zr_select_workspace_bytes(0) == 0 && zr_select_workspace_bytes(1000) == 0 && zr_select_workspace_bytes(1 << 20) > 0);
    EXPECT(zr_resize_select_ws(nullptr, 8, 0.25, KI, KI, P, 1 << 20, nullptr) == ZR_ERR_NULL);
    EXPECT(zr_resize_select_ws(SC, 0, 0.25, KI, KI, P, 1 << 20, nullptr) == ZR_ERR_SHAPE);
    EXPECT(zr_resize_select_ws(SC, (1 << 24) + 1, 0.25, KI, KI, P, 1 << 20, nullptr) == ZR_ERR_LIMIT);
    EXPECT(zr_resize_select_ws(SC, 8, 1.0, KI, KI, P, 1 << 20, nullptr) == ZR_ERR_RATIO);
    EXPECT(zr_resize_select_ws(SC, 8, 0.25, KI, nullptr, nullptr, 0, nullptr) == ZR_OK);
    EXPECT(zr_resize_select_ws(SC, 1 << 20, 0.25, KI, KI, P, 16, nullptr) == ZR_OK);
    EXPECT(zr_resize_select_ws(SC, 1 << 20, 0.25, KI, KI, P, zr_select_workspace_bytes(1 << 20), nullptr) == ZR_OK);
    {
        const float* sc[17]; int32_t n[17]; double r[17]; int32_t* k[17]; int32_t* d[17];
        for (int b = 0; b < 17; ++b) { sc[b] = SC; n[b] = 16 + b; r[b] = 0.1 * (b % 5); k[b] = KI; d[b] = b % 2 ? KI : nullptr; }
        EXPECT(zr_resize_select_multi(0, sc, n, r, k, d, nullptr) == ZR_ERR_SHAPE);
        EXPECT(zr_resize_select_multi(17, sc, n, r, k, d, nullptr) == ZR_ERR_LIMIT);
        EXPECT(zr_resize_select_multi(16, sc, n, r, k, d, nullptr) == ZR_OK && zr_resize_select_multi(5, sc, n, r, k, nullptr, nullptr) == ZR_OK);
        sc[3] = nullptr; EXPECT(zr_resize_select_multi(5, sc, n, r, k, d, nullptr) == ZR_ERR_NULL); sc[3] = SC;
        n[2] = 0; EXPECT(zr_resize_select_multi(5, sc, n, r, k, d, nullptr) == ZR_ERR_SHAPE); n[2] = 18;
        r[1] = 1.5; EXPECT(zr_resize_select_multi(5, sc, n, r, k, d, nullptr) == ZR_ERR_RATIO);
        EXPECT(zr_resize_select_multi(5, nullptr, n, r, k, d, nullptr) == ZR_ERR_NULL);
    }

    // ---- forward / backward: bad arguments
    const int M = 96, K = 136, N = 200;
    EXPECT(zr_resized_linear_fwd(nullptr, K, P, N, P, N, M, K, N, KI, 8, ZR_DROP_N, ZR_W_KN, ZR_BF16, ZR_IMPUTE_ZERO, nullptr, nullptr, 0, nullptr) == ZR_ERR_NULL);
    EXPECT(zr_resized_linear_fwd(P, K, P, N, P, N, M, K, N, nullptr, 8, ZR_DROP_N, ZR_W_KN, ZR_BF16, ZR_IMPUTE_ZERO, nullptr, nullptr, 0, nullptr) == ZR_ERR_NULL);
    EXPECT(zr_resized_linear_fwd(P, K, P, N, P, N, M, K, N, KI, 8, ZR_DROP_N, ZR_W_KN, 7, ZR_IMPUTE_ZERO, nullptr, nullptr, 0, nullptr) == ZR_ERR_DTYPE);
    EXPECT(zr_resized_linear_fwd(P, K, P, N, P, N, M, K, N, KI, 8, 5, ZR_W_KN, ZR_BF16, ZR_IMPUTE_ZERO, nullptr, nullptr, 0, nullptr) == ZR_ERR_MODE);
    EXPECT(zr_resized_linear_fwd(P, K, P, N, P, N, M, K, N, KI, 8, ZR_DROP_N, 9, ZR_BF16, ZR_IMPUTE_ZERO, nullptr, nullptr, 0, nullptr) == ZR_ERR_MODE);
    EXPECT(zr_resized_linear_fwd(P, K, P, N, P, N, M, K, N, KI, 8, ZR_DROP_N, ZR_W_KN, ZR_BF16, 3, nullptr, nullptr, 0, nullptr) == ZR_ERR_POLICY);
    EXPECT(zr_resized_linear_fwd(P, K, P, N, P, N, 0, K, N, KI, 8, ZR_DROP_N, ZR_W_KN, ZR_BF16, ZR_IMPUTE_ZERO, nullptr, nullptr, 0, nullptr) == ZR_ERR_SHAPE);
    EXPECT(zr_resized_linear_fwd(P, K, P, N, P, N, M, K, N, KI, 0, ZR_DROP_N, ZR_W_KN, ZR_BF16, ZR_IMPUTE_ZERO, nullptr, nullptr, 0, nullptr) == ZR_ERR_INDEX);
    EXPECT(zr_resized_linear_fwd(P, K, P, N, P, N, M, K, N, KI, N + 1, ZR_DROP_N, ZR_W_KN, ZR_BF16, ZR_IMPUTE_ZERO, nullptr, nullptr, 0, nullptr) == ZR_ERR_INDEX);
    EXPECT(zr_resized_linear_fwd(P, K, P, N, P, N, M, K, N, KI, K + 1, ZR_DROP_K, ZR_W_KN, ZR_BF16, ZR_IMPUTE_ZERO, nullptr, nullptr, 0, nullptr) == ZR_ERR_INDEX);
    EXPECT(zr_resized_linear_fwd(P, K - 1, P, N, P, N, M, K, N, KI, 8, ZR_DROP_N, ZR_W_KN, ZR_BF16, ZR_IMPUTE_ZERO, nullptr, nullptr, 0, nullptr) == ZR_ERR_SHAPE);
    EXPECT(zr_resized_linear_fwd(P, K, P, N - 1, P, N, M, K, N, KI, 8, ZR_DROP_N, ZR_W_KN, ZR_BF16, ZR_IMPUTE_ZERO, nullptr, nullptr, 0, nullptr) == ZR_ERR_SHAPE);
    EXPECT(zr_resized_linear_fwd(P, K, P, K - 1, P, N, M, K, N, KI, 8, ZR_DROP_N, ZR_W_NK, ZR_BF16, ZR_IMPUTE_ZERO, nullptr, nullptr, 0, nullptr) == ZR_ERR_SHAPE);
    EXPECT(zr_resized_linear_fwd(P, K, P, N, P, N - 1, M, K, N, KI, 8, ZR_DROP_N, ZR_W_KN, ZR_BF16, ZR_IMPUTE_ZERO, nullptr, nullptr, 0, nullptr) == ZR_ERR_SHAPE);
    EXPECT(zr_resized_linear_fwd(P, K, P, N, P, N, M, K, N, KI, 8, ZR_DROP_N, ZR_W_KN, ZR_BF16, ZR_IMPUTE_SAME, nullptr, nullptr, 0, nullptr) == ZR_ERR_POLICY);
    EXPECT(zr_resized_linear_bwd(P, K, P, N, nullptr, N, P, K, P, N, M, K, N, KI, 8, ZR_DROP_N, ZR_W_KN, ZR_BF16, ZR_IMPUTE_ZERO, nullptr, nullptr, nullptr, 0, 0, nullptr) == ZR_ERR_NULL);
    EXPECT(zr_resized_linear_bwd(P, K, P, N, P, N, nullptr, K, nullptr, N, M, K, N, KI, 8, ZR_DROP_N, ZR_W_KN, ZR_BF16, ZR_IMPUTE_ZERO, nullptr, nullptr, nullptr, 0, 0, nullptr) == ZR_ERR_NULL);
    EXPECT(zr_resized_linear_bwd(P, K, nullptr, N, P, N, P, K, nullptr, N, M, K, N, KI, 8, ZR_DROP_N, ZR_W_KN, ZR_BF16, ZR_IMPUTE_ZERO, nullptr, nullptr, nullptr, 0, 0, nullptr) == ZR_ERR_NULL);
    EXPECT(zr_resized_linear_bwd(nullptr, K, P, N, P, N, nullptr, K, P, N, M, K, N, KI, 8, ZR_DROP_N, ZR_W_KN, ZR_BF16, ZR_IMPUTE_ZERO, nullptr, nullptr, nullptr, 0, 0, nullptr) == ZR_ERR_NULL);
    EXPECT(zr_resized_linear_bwd(P, K, P, N, P, N - 1, P, K, P, N, M, K, N, KI, 8, ZR_DROP_N, ZR_W_KN, ZR_BF16, ZR_IMPUTE_ZERO, nullptr, nullptr, nullptr, 0, 0, nullptr) == ZR_ERR_SHAPE);
    EXPECT(zr_resized_linear_bwd(P, K, P, N, P, N, P, K - 1, P, N, M, K, N, KI, 8, ZR_DROP_N, ZR_W_KN, ZR_BF16, ZR_IMPUTE_ZERO, nullptr, nullptr, nullptr, 0, 0, nullptr) == ZR_ERR_SHAPE);
    EXPECT(zr_resized_linear_bwd(P, K, P, N, P, N, P, K, P, N - 1, M, K, N, KI, 8, ZR_DROP_N, ZR_W_KN, ZR_BF16, ZR_IMPUTE_ZERO, nullptr, nullptr, nullptr, 0, 0, nullptr) == ZR_ERR_SHAPE);
    EXPECT(zr_resized_linear_bwd(P, K, P, N, P, N, P, K, P, N, M, K, N, KI, 8, ZR_DROP_K, ZR_W_KN, ZR_BF16, ZR_IMPUTE_SAME, nullptr, P, nullptr, 0, 0, nullptr) == ZR_ERR_POLICY);
    EXPECT(zr_resized_linear_bwd(P, K, P, N, P, N, P, K, P, N, M, K, N, KI, 8, ZR_DROP_K, ZR_W_KN, ZR_BF16, ZR_IMPUTE_SAME, P, nullptr, nullptr, 0, 0, nullptr) == ZR_ERR_POLICY);

    // ---- forward / backward: every mode x layout x policy x dtype, kept counts from 1 to all,
    // workspaces of every awkward size (the calls carve the sums from the tail, the extraction
    // from the head and the split scratch from between; the stubs check the placement)
    std::vector<char> wsbuf((size_t)80 << 20);
    char* ws0 = (char*)(((uintptr_t)wsbuf.data() + 15) & ~(uintptr_t)15);
    int ok_calls = 0;
    for (int dtype : {ZR_F32, ZR_BF16})
        for (int mode : {ZR_DROP_N, ZR_DROP_K})
            for (int layout : {ZR_W_KN, ZR_W_NK})
                for (int policy : {ZR_IMPUTE_ZERO, ZR_IMPUTE_AVERAGE, ZR_IMPUTE_SAME}) {
                    const int n = mode == ZR_DROP_N ? N : K;
                    const int64_t ldw = layout == ZR_W_KN ? N : K;
                    for (int n_keep : {1, 2, n / 2, n - 1, n}) {
                        const size_t full = zr_workspace_bytes(M, K, N, n_keep, mode, dtype);
                        for (size_t bytes : {(size_t)0, (size_t)1, (size_t)15, (size_t)16, (size_t)17, (size_t)M * 64 * 2, full / 2, full - 1, full, full + 13}) {
                            for (int misalign : {0, 4}) {
                                void* ws = bytes ? ws0 + misalign : nullptr;
                                if (bytes + misalign > ((size_t)79 << 20)) continue;
                                zr::g_ws_begin = (const char*)ws; zr::g_ws_end = (const char*)ws + bytes;
                                int st = zr_resized_linear_fwd(P, K, P, ldw, P, N, M, K, N, KI, n_keep, mode, layout, dtype, policy, P, ws, bytes, nullptr);
                                EXPECT(st == ZR_OK);
                                for (int flags : {0, 1}) {
                                    st = zr_resized_linear_bwd(P, K, P, ldw, P, N, P, K, P, ldw, M, K, N, KI, n_keep, mode, layout, dtype, policy, P, P, ws, bytes, flags, nullptr);
                                    EXPECT(st == ZR_OK);
                                    st = zr_resized_linear_bwd(nullptr, K, P, ldw, P, N, P, K, nullptr, ldw, M, K, N, KI, n_keep, mode, layout, dtype, policy, P, P, ws, bytes, flags, nullptr);
                                    EXPECT(st == ZR_OK);
                                    st = zr_resized_linear_bwd(P, K, nullptr, ldw, P, N, nullptr, K, P, ldw, M, K, N, KI, n_keep, mode, layout, dtype, policy, P, P, ws, bytes, flags, nullptr);
                                    EXPECT(st == ZR_OK);
                                }
                                ok_calls += 7;
                            }
                        }
                    }
                }
    zr::g_ws_begin = zr::g_ws_end = nullptr;

    // ---- the other device entry points
    EXPECT(zr_extract_kept_columns(nullptr, 8, 4, 8, KI, 4, P, 64, ZR_BF16, nullptr) == ZR_ERR_NULL);
    EXPECT(zr_extract_kept_columns(P, 8, 4, 8, KI, 4, P, 64, ZR_F32, nullptr) == ZR_ERR_DTYPE);
    EXPECT(zr_extract_kept_columns(P, 6, 4, 8, KI, 4, P, 64, ZR_BF16, nullptr) == ZR_ERR_SHAPE);
    EXPECT(zr_extract_kept_columns(P, 8, 4, 8, KI, 9, P, 64, ZR_BF16, nullptr) == ZR_ERR_INDEX);
    EXPECT(zr_extract_kept_columns(P, 8, 4, 8, KI, 4, P, 32, ZR_BF16, nullptr) == ZR_ERR_SHAPE);
    EXPECT(zr_extract_kept_columns(P, 8, 4, 8, KI, 4, (char*)P + 2, 64, ZR_BF16, nullptr) == ZR_ERR_SHAPE);
    EXPECT(zr_extract_kept_columns(P, 8, 4, 8, KI, 4, P, 64, ZR_BF16, nullptr) == ZR_OK);
    EXPECT(zr_impute(nullptr, 8, 4, 8, 1, KI, 4, ZR_IMPUTE_ZERO, nullptr, ZR_BF16, nullptr) == ZR_ERR_NULL);
    EXPECT(zr_impute(P, 8, 4, 8, 2, KI, 4, ZR_IMPUTE_ZERO, nullptr, ZR_BF16, nullptr) == ZR_ERR_SHAPE);
    EXPECT(zr_impute(P, 7, 4, 8, 1, KI, 4, ZR_IMPUTE_ZERO, nullptr, ZR_BF16, nullptr) == ZR_ERR_SHAPE);
    EXPECT(zr_impute(P, 8, 4, 8, 0, KI, 5, ZR_IMPUTE_ZERO, nullptr, ZR_BF16, nullptr) == ZR_ERR_INDEX);
    EXPECT(zr_impute(P, 8, 4, 8, 1, KI, 4, ZR_IMPUTE_SAME, nullptr, ZR_BF16, nullptr) == ZR_ERR_POLICY);
    EXPECT(zr_impute(P, 8, (1 << 21) + 1, 8, 1, KI, 4, ZR_IMPUTE_ZERO, nullptr, ZR_BF16, nullptr) == ZR_ERR_LIMIT);
    // 32 rows per workgroup of a grid dimension that holds 65535: the last size that fits, and the first that does not
    EXPECT(zr_impute(P, 8, 65535 * 32 + 1, 8, 1, KI, 4, ZR_IMPUTE_ZERO, nullptr, ZR_BF16, nullptr) == ZR_ERR_LIMIT);
    EXPECT(zr_resized_linear_fwd(P, 8, P, 8, P, 8, 65535 * 32 + 1, 8, 8, KI, 4, ZR_DROP_K, ZR_W_KN, ZR_BF16, ZR_IMPUTE_ZERO,
                                 nullptr, nullptr, 0, nullptr) == ZR_ERR_LIMIT);
    EXPECT(zr_impute(P, 8, 4, 8, 1, KI, 4, ZR_IMPUTE_AVERAGE, nullptr, ZR_F32, nullptr) == ZR_OK);
    EXPECT(zr_priority_scores(nullptr, P, 8, 4, 8, ZR_DROP_N, nullptr, nullptr, 0, SC, ZR_BF16, nullptr, 0, nullptr) == ZR_ERR_NULL);
    EXPECT(zr_priority_scores(P, P, 7, 4, 8, ZR_DROP_N, nullptr, nullptr, 0, SC, ZR_BF16, nullptr, 0, nullptr) == ZR_ERR_SHAPE);
    EXPECT(zr_priority_scores(P, P, 8, 4, 8, ZR_DROP_N, nullptr, KI, 3, SC, ZR_BF16, nullptr, 0, nullptr) == ZR_ERR_NULL);
    EXPECT(zr_priority_scores(P, P, 8, 4, 8, ZR_DROP_N, SC, KI, 9, SC, ZR_BF16, nullptr, 0, nullptr) == ZR_ERR_INDEX);
    EXPECT(zr_priority_scores(P, P, 8, 4, 8, ZR_DROP_K, SC, KI, 4, SC, ZR_F32, nullptr, 0, nullptr) == ZR_OK);
    EXPECT(zr_priority_scores_static(P, P, 8, 4, 8, ZR_DROP_N, SC, KI, 4, SC, ZR_BF16, nullptr) == ZR_OK);
    EXPECT(zr_priority_scores_static(P, P, 400000, 4, 400000, ZR_DROP_N, nullptr, nullptr, 0, SC, ZR_BF16, nullptr) == ZR_ERR_LIMIT);
    EXPECT(zr_priority_scores_static(P, P, 8, 4, 8, 3, nullptr, nullptr, 0, SC, ZR_BF16, nullptr) == ZR_ERR_MODE);
    EXPECT(zr_count_above(nullptr, 4, 0.5f, KI, nullptr) == ZR_ERR_NULL && zr_count_above(SC, 0, 0.5f, KI, nullptr) == ZR_ERR_SHAPE && zr_count_above(SC, 4, 0.5f, KI, nullptr) == ZR_OK);
    EXPECT(zr_migrated_accumulate(P, 8, P, 8, 0, nullptr, 8, 4, 8, 8, ZR_BF16, nullptr) == ZR_ERR_NULL);
    EXPECT(zr_migrated_accumulate(P, 7, P, 8, 0, P, 8, 4, 8, 8, ZR_BF16, nullptr) == ZR_ERR_SHAPE);
    EXPECT(zr_migrated_accumulate(P, 8, P, 7, 1, P, 8, 4, 8, 8, ZR_BF16, nullptr) == ZR_ERR_SHAPE);
    EXPECT(zr_migrated_accumulate(P, 8, P, 8, 1, P, 8, 4, 8, 8, ZR_F32, nullptr) == ZR_OK);
    EXPECT(zr_validate_keep_idx(nullptr, 4, 8, KI, nullptr) == ZR_ERR_NULL && zr_validate_keep_idx(KI, 9, 8, KI, nullptr) == ZR_ERR_INDEX && zr_validate_keep_idx(KI, 4, 8, KI, nullptr) == ZR_OK);
    double fl = 0;
    EXPECT(zr_debug_mfma_rate(0, 1, SC, &fl, nullptr) == ZR_ERR_SHAPE && zr_debug_mfma_rate(2, 3, nullptr, &fl, nullptr) == ZR_ERR_NULL);
    EXPECT(zr_debug_mfma_rate(2, 3, SC, &fl, nullptr) == ZR_OK && fl == 12.0);
    EXPECT(zr_debug_time_next_product(nullptr, P) == ZR_ERR_NULL);
    zr_debug_record_kernel_names(1); zr_debug_record_kernel_names(0);
    EXPECT(zr_debug_last_kernel() != nullptr);

    printf("%s: %d checked calls with good arguments, %d launches seen by the stubs, %d failures\n",
           failures ? "FAILED" : "OK", ok_calls, zr::g_launches, failures);
    return failures ? 1 : 0;
}

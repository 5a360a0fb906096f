// Internal declarations shared by the HIP translation units of libzr.
// Written for gfx950 (MI355X) only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>

#include "zr.h"
#include "zr_debug.h"

namespace zr {

// ---- bf16 <-> fp32 on raw 16-bit storage -----------------------------------
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h)
{
    return __uint_as_float(h << 16);
}

// round-to-nearest-even; NaN stays NaN (quietened)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// clamp an index read from a caller's list into [0, n): a malformed list may
// give wrong values but never an out-of-range access
__device__ __forceinline__ int clamp_idx(int v, int n)
{
    return v < 0 ? 0 : (v >= n ? n - 1 : v);
}

// ---- problem description handed from the C ABI to the GEMM launcher ---------
//
// Every product is brought to the canonical form
//     D[i, j] = sum_c A(i, c) * B(j, c),   i < I, j < J, c < C
// where each operand is addressed as base[rowmap(r) * ld + colmap(q)] with r the
// index along the tensor's strided axis and q along its contiguous axis; either
// map may be absent (identity) or the kept-index list.
struct Operand {
    const void* base;
    int64_t ld;          // elements
    // which canonical index runs along the tensor's contiguous axis
    // true : contraction index c is contiguous  ("format P", e.g. X in Y = X W)
    // false: the non-contraction index is contiguous ("format Q", e.g. W in Y = X W)
    bool c_contig;
    const int32_t* map_strided;   // list applied to the strided axis, or nullptr
    const int32_t* map_contig;    // list applied to the contiguous axis, or nullptr
    int n_strided;                // full extent of the strided axis in memory (for clamping)
    int n_contig;                 // readable extent of the contiguous axis in memory
    // the tensor holds real zeros from the end of its logical extent up to the next
    // multiple of 64 along the contiguous axis (extracted activations in the workspace)
    bool zero_padded;
};

enum Epilogue { EPI_PLAIN = 0, EPI_COL_SCATTER = 1, EPI_ROW_SCATTER = 2 };

struct GemmDesc {
    Operand A, B;
    int I, J, C;
    void* out;
    int64_t ldo;
    int epilogue;
    const int32_t* keep_idx;   // list used by the scatter epilogues
    int out_full;              // full extent of the scattered output axis
    int dtype;
    // Same imputation fused into the scatter epilogues: dropped positions copy this
    // tensor (laid out like `out`, may alias it) instead of receiving +0
    const void* prev = nullptr;
    // out = round(out + D) in fp32 (plain epilogue only): the local reduce of migrated work
    bool accumulate = false;
    // Average imputation, first phase (scatter epilogues only): every tile adds up the
    // results it stores, per output row over its columns (column scatter) or per output
    // column over its rows (row scatter), and writes the sums to
    // avg_partial[slot * avg_len + index], slot = the tile's position along the summed
    // axis.  The buffer holds ceil(extent / 128) slots and must be zero beforehand.
    float* avg_partial = nullptr;
    int avg_len = 0;
    // Scratch for a split contraction (16-byte aligned; products with too few tiles to fill the
    // chip cut the contraction into slices and add them up in a second launch); nullptr: never split.
    void* split_scratch = nullptr;
    size_t split_scratch_bytes = 0;
};

// State of the aids in zr_debug.h, per host thread.  Product calls only test `armed`.
struct DebugState {
    bool record_names = false;      // zr_debug_record_kernel_names
    bool armed_once = false;        // zr_debug_time_next_product: name + events for the next product
    hipEvent_t start = nullptr, stop = nullptr;
    char last_kernel[128] = "";
};
extern thread_local DebugState g_debug;
inline bool debug_names_wanted() { return g_debug.record_names || g_debug.armed_once; }

// Dynamic-LDS attribute of a kernel: set once per device and instantiation (the call is
// idempotent, so two threads racing to set it do no harm; the flags are atomic).
struct AttrFlags {
    static constexpr int MAX_DEVICES = 16;
    std::atomic<bool> done[MAX_DEVICES] = {};
};
bool ensure_max_dynamic_lds(const void* fn, int bytes, void* flags16);
int launch_gemm(const GemmDesc& d, hipStream_t stream);
int launch_gemm_fast(const GemmDesc& d, hipStream_t stream);   // -1: not eligible
int launch_select(const float* scores, int n, int batch, int n_keep,
                  int32_t* keep_idx, int32_t* drop_idx, int64_t ld_idx, hipStream_t stream);
// one long vector on many workgroups, with caller scratch of select_wide_workspace_bytes()
size_t select_wide_workspace_bytes();
int select_wide_min_n();
int launch_select_wide(const float* scores, int n, int n_keep, int32_t* keep_idx, int32_t* drop_idx,
                       void* workspace, hipStream_t stream);
constexpr int ZR_SELECT_MULTI_MAX = 16;
struct SelectMulti {
    const float* scores[ZR_SELECT_MULTI_MAX];
    int32_t* keep[ZR_SELECT_MULTI_MAX];
    int32_t* drop[ZR_SELECT_MULTI_MAX];
    int n[ZR_SELECT_MULTI_MAX];
    int n_keep[ZR_SELECT_MULTI_MAX];
};
int launch_select_multi(const SelectMulti& m, int count, hipStream_t stream);
int launch_impute(void* out, int64_t ld, int rows, int cols, int axis,
                  const int32_t* keep_idx, int n_keep, int policy, const void* prev,
                  int dtype, hipStream_t stream);
// Average imputation, second phase: mean[i] = (sum over slots of partial[slot*len + i]) / n_keep
// (in slot order, left in slot 0), then the dropped columns / rows receive the mean.
int launch_zero_f32(float* p, size_t count, hipStream_t stream);
int launch_mean_fill(void* out, int64_t ld, int rows, int cols, int axis, const int32_t* keep_idx, int n_keep,
                     float* partial, int slots, int dtype, hipStream_t stream);
int launch_compact_cols(const void* in, int64_t ld, int rows, int n, const int32_t* keep, int n_keep,
                        void* out, int64_t ldo, int width, hipStream_t stream);
int launch_priority_scores(const void* Wt, const void* Wp, int64_t ld, int K, int N, int mode,
                           const float* prev_scores, const int32_t* prev_keep, int n_prev_keep,
                           float* scores, int dtype, void* workspace, size_t workspace_bytes, hipStream_t stream);
size_t priority_workspace_bytes(int K, int N, int mode);
int launch_priority_scores_static(const void* Wt, const void* Wp, int64_t ld, int K, int N, int mode,
                                  const float* prev_scores, const int32_t* prev_keep, int n_prev_keep,
                                  float* scores, int dtype, hipStream_t stream);
size_t priority_static_scratch_bytes();
int launch_count_above(const float* scores, int n, float theta, int32_t* count, hipStream_t stream);
int launch_mfma_rate(int blocks, int iters, float* sink, hipStream_t stream);   // zr_probe.hip
double mfma_rate_flops(int blocks, int iters);
int launch_validate(const int32_t* keep_idx, int n_keep, int n, int32_t* flag, hipStream_t stream);

inline int hip_status(hipError_t e) { return e == hipSuccess ? ZR_OK : ZR_ERR_HIP; }

}  // namespace zr

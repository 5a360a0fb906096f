// Priority bookkeeping of ZERO-resizing (paper Sec. 3.2 and Algorithm 1, the
// per-layer block that precedes the top-L_pri select):
//   delta_i = (1/R) * sum_j |w_ji^t - w_ji^(t-1)|   weight variation of slice i
//   an index pruned in the previous epoch keeps its previous score (incremental update)
//   L_uni   = #{ i : delta_i > theta }                (differentiated per-layer ratio)
// HBM-bound reductions over the two weight snapshots; every sum is taken in a
// fixed order (no floating-point atomics), so results are bitwise repeatable.
#include <atomic>

#include "zr_common.h"

namespace zr {

namespace {

// Scratch of zr_priority_scores_static: the per-row-range column sums that the ordinary
// entry point keeps in the caller's workspace.  One copy per GPU the library runs on, held
// until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels are always given the address that call returned.
constexpr size_t kStaticScratchBytes = (size_t)1 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 16;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device (looked up once per device).
int static_scratch(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ZR_ERR_HIP;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return ZR_ERR_HIP;
        g_scratch_ptr[dev].store(p, std::memory_order_release);     // every thread finds the same address
    }
    *out = p;
    return ZR_OK;
}

template <typename T, int V> struct Vec;
template <> struct Vec<float, 1>    { using type = float; };
template <> struct Vec<float, 4>    { using type = float4; };
template <> struct Vec<uint16_t, 1> { using type = uint16_t; };
template <> struct Vec<uint16_t, 4> { using type = uint2; };
template <> struct Vec<uint16_t, 8> { using type = uint4; };

__device__ __forceinline__ float absdiff(float a, float b) { return fabsf(a - b); }

// |a - b| of V consecutive elements, added element-wise into acc[V]
template <typename T, int V>
__device__ __forceinline__ void accum(const T* __restrict__ a, const T* __restrict__ b, float* acc)
{
    using VT = typename Vec<T, V>::type;
    const VT va = *reinterpret_cast<const VT*>(a);
    const VT vb = *reinterpret_cast<const VT*>(b);
    if constexpr (sizeof(T) == 4) {
        const float* pa = reinterpret_cast<const float*>(&va);
        const float* pb = reinterpret_cast<const float*>(&vb);
#pragma unroll
        for (int i = 0; i < V; ++i) acc[i] += absdiff(pa[i], pb[i]);
    } else if constexpr (V == 1) {
        acc[0] += absdiff(bf16_bits_to_f32(va), bf16_bits_to_f32(vb));
    } else {
        const uint32_t* pa = reinterpret_cast<const uint32_t*>(&va);
        const uint32_t* pb = reinterpret_cast<const uint32_t*>(&vb);
#pragma unroll
        for (int i = 0; i < V / 2; ++i) {
            acc[2 * i]     += absdiff(__uint_as_float(pa[i] << 16), __uint_as_float(pb[i] << 16));
            acc[2 * i + 1] += absdiff(__uint_as_float(pa[i] & 0xffff0000u), __uint_as_float(pb[i] & 0xffff0000u));
        }
    }
}

// true if p is in the ascending list keep[0..n_keep)
__device__ __forceinline__ bool in_list(const int32_t* __restrict__ keep, int n_keep, int p)
{
    int lo = 0, hi = n_keep;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (keep[mid] < p) lo = mid + 1; else hi = mid;
    }
    return lo < n_keep && keep[lo] == p;
}

__device__ __forceinline__ float finish(float sum, int R, int idx, const float* __restrict__ prev_scores,
                                        const int32_t* __restrict__ prev_keep, int n_prev_keep)
{
    if (prev_keep && !in_list(prev_keep, n_prev_keep, idx)) return prev_scores[idx];
    return sum / (float)R;
}

// Column sums of |W_t - W_prev| over the rows [blockIdx.y * rows_per, +rows_per).
// A lane owns V adjacent columns, a workgroup 64*V columns; its 16 wavefronts
// take rows w, w+16, ... and their partial sums are added in wavefront order.
// FINAL: the grid has one row range and writes the scores; otherwise it writes
// the range's sums to partial[blockIdx.y][N].
template <typename T, int V, bool FINAL>
__global__ __launch_bounds__(1024) void col_sums_kernel(
    const T* __restrict__ Wt, const T* __restrict__ Wp, int64_t ld, int K, int N, int rows_per,
    const float* __restrict__ prev_scores, const int32_t* __restrict__ prev_keep, int n_prev_keep,
    float* __restrict__ out)
{
    __shared__ float part[16][64 * V];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = (blockIdx.x * 64 + lane) * V;
    const int r0 = blockIdx.y * rows_per;
    const int r1 = min(K, r0 + rows_per);
    float acc[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.f;
    if (col < N) {                      // V > 1 is only launched with N % V == 0
        const size_t step = (size_t)ld * 16;
        size_t off = (size_t)(r0 + wave) * (size_t)ld + (size_t)col;
        int r = r0 + wave;
        for (; r + 48 < r1; r += 64, off += 4 * step) {
            accum<T, V>(Wt + off, Wp + off, acc);
            accum<T, V>(Wt + off + step, Wp + off + step, acc);
            accum<T, V>(Wt + off + 2 * step, Wp + off + 2 * step, acc);
            accum<T, V>(Wt + off + 3 * step, Wp + off + 3 * step, acc);
        }
        for (; r < r1; r += 16, off += step) accum<T, V>(Wt + off, Wp + off, acc);
    }
#pragma unroll
    for (int i = 0; i < V; ++i) part[wave][lane * V + i] = acc[i];
    __syncthreads();
    for (int t = threadIdx.x; t < 64 * V; t += 1024) {
        const int c = blockIdx.x * 64 * V + t;
        if (c >= N) continue;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < 16; ++w) sum += part[w][t];
        if (FINAL) out[c] = finish(sum, K, c, prev_scores, prev_keep, n_prev_keep);
        else       out[(size_t)blockIdx.y * (size_t)N + c] = sum;
    }
}

// scores[c] from the per-range sums partial[n_split][N], added in range order
__global__ __launch_bounds__(256) void col_finish_kernel(
    const float* __restrict__ partial, int n_split, int K, int N,
    const float* __restrict__ prev_scores, const int32_t* __restrict__ prev_keep, int n_prev_keep,
    float* __restrict__ scores)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= N) return;
    float sum = 0.f;
    for (int s = 0; s < n_split; ++s) sum += partial[(size_t)s * (size_t)N + c];
    scores[c] = finish(sum, K, c, prev_scores, prev_keep, n_prev_keep);
}

// Scores of the ROWS of W[K x N] (pruned axis = K): one wavefront per row, a
// lane adds its elements in column order, then a fixed shuffle tree.
template <typename T, int V>
__global__ __launch_bounds__(256) void row_scores_kernel(
    const T* __restrict__ Wt, const T* __restrict__ Wp, int64_t ld, int K, int N,
    const float* __restrict__ prev_scores, const int32_t* __restrict__ prev_keep, int n_prev_keep,
    float* __restrict__ scores)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= K) return;
    const T* a = Wt + (size_t)row * (size_t)ld;
    const T* b = Wp + (size_t)row * (size_t)ld;
    float acc[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.f;
    int c = lane * V;                   // V > 1 is only launched with N % V == 0
    for (; c + 3 * 64 * V < N; c += 4 * 64 * V) {
        accum<T, V>(a + c, b + c, acc);
        accum<T, V>(a + c + 64 * V, b + c + 64 * V, acc);
        accum<T, V>(a + c + 2 * 64 * V, b + c + 2 * 64 * V, acc);
        accum<T, V>(a + c + 3 * 64 * V, b + c + 3 * 64 * V, acc);
    }
    for (; c < N; c += 64 * V) accum<T, V>(a + c, b + c, acc);
    float sum = acc[0];
#pragma unroll
    for (int i = 1; i < V; ++i) sum += acc[i];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_down(sum, off, 64);
    if (lane == 0) scores[row] = finish(sum, N, row, prev_scores, prev_keep, n_prev_keep);
}

__global__ __launch_bounds__(1024) void count_above_kernel(const float* __restrict__ scores, int n, float theta,
                                                           int32_t* __restrict__ count)
{
    __shared__ int wsum[16];
    int c = 0;
    for (int i = threadIdx.x; i < n; i += 1024) c += scores[i] > theta ? 1 : 0;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) c += __shfl_down(c, off, 64);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = 0;
        for (int w = 0; w < 16; ++w) t += wsum[w];
        *count = t;
    }
}

#ifndef ZR_PRI_BLOCKS
#define ZR_PRI_BLOCKS 256               // one workgroup of 16 wavefronts per compute unit measured fastest
#endif
#ifndef ZR_PRI_MIN_ROWS
#define ZR_PRI_MIN_ROWS 256
#endif
constexpr int kTargetBlocks = ZR_PRI_BLOCKS;
constexpr int kMinRowsPerSplit = ZR_PRI_MIN_ROWS;

template <int V> int col_splits(int K, int N)
{
    const int chunks = (N + 64 * V - 1) / (64 * V);
    const int by_rows = (K + kMinRowsPerSplit - 1) / kMinRowsPerSplit;
    const int want = (kTargetBlocks + chunks - 1) / chunks;
    return std::max(1, std::min(by_rows, want));
}

template <typename T, int V>
int cols_typed(const T* Wt, const T* Wp, int64_t ld, int K, int N, const float* prev_scores,
               const int32_t* prev_keep, int n_prev_keep, float* scores, void* workspace, size_t workspace_bytes,
               hipStream_t stream)
{
    const int chunks = (N + 64 * V - 1) / (64 * V);
    int splits = col_splits<V>(K, N);
    const size_t fit = workspace ? workspace_bytes / ((size_t)N * sizeof(float)) : 0;   // row ranges the scratch holds
    if ((size_t)splits > fit) splits = fit < 2 ? 1 : (int)fit;
    if (splits == 1) {
        hipLaunchKernelGGL((col_sums_kernel<T, V, true>), dim3(chunks, 1), dim3(1024), 0, stream,
                           Wt, Wp, ld, K, N, K, prev_scores, prev_keep, n_prev_keep, scores);
        return hip_status(hipGetLastError());
    }
    const int rows_per = (((K + splits - 1) / splits) + 15) & ~15;
    splits = (K + rows_per - 1) / rows_per;
    float* partial = (float*)workspace;
    hipLaunchKernelGGL((col_sums_kernel<T, V, false>), dim3(chunks, splits), dim3(1024), 0, stream,
                       Wt, Wp, ld, K, N, rows_per, prev_scores, prev_keep, n_prev_keep, partial);
    hipLaunchKernelGGL(col_finish_kernel, dim3((N + 255) / 256), dim3(256), 0, stream,
                       partial, splits, K, N, prev_scores, prev_keep, n_prev_keep, scores);
    return hip_status(hipGetLastError());
}

template <typename T, int V>
int rows_typed(const T* Wt, const T* Wp, int64_t ld, int K, int N, const float* prev_scores,
               const int32_t* prev_keep, int n_prev_keep, float* scores, hipStream_t stream)
{
    hipLaunchKernelGGL((row_scores_kernel<T, V>), dim3((K + 3) / 4), dim3(256), 0, stream,
                       Wt, Wp, ld, K, N, prev_scores, prev_keep, n_prev_keep, scores);
    return hip_status(hipGetLastError());
}

// widest vector (in elements) both snapshots allow for every row start
template <typename T> int vec_width(const T* Wt, const T* Wp, int64_t ld, int N, int vmax)
{
    for (int v = vmax; v > 1; v >>= 1) {
        const uintptr_t bytes = (uintptr_t)v * sizeof(T);
        if (N % v == 0 && ld % v == 0 && (uintptr_t)Wt % bytes == 0 && (uintptr_t)Wp % bytes == 0) return v;
    }
    return 1;
}

}  // namespace

size_t priority_workspace_bytes(int K, int N, int mode)
{
    if (mode != ZR_DROP_N) return 0;
    // the widest column chunk leaves the fewest chunks, hence the most row ranges
    return (size_t)std::max(col_splits<1>(K, N), col_splits<4>(K, N)) * (size_t)N * sizeof(float);
}

int launch_priority_scores(const void* Wt, const void* Wp, int64_t ld, int K, int N, int mode,
                           const float* prev_scores, const int32_t* prev_keep, int n_prev_keep,
                           float* scores, int dtype, void* workspace, size_t workspace_bytes, hipStream_t stream)
{
#define ZR_ARGS(T) (const T*)Wt, (const T*)Wp, ld, K, N, prev_scores, prev_keep, n_prev_keep, scores
    if (dtype == ZR_F32) {
        const int v = vec_width((const float*)Wt, (const float*)Wp, ld, N, 4);
        if (mode == ZR_DROP_N)
            return v == 4 ? cols_typed<float, 4>(ZR_ARGS(float), workspace, workspace_bytes, stream)
                          : cols_typed<float, 1>(ZR_ARGS(float), workspace, workspace_bytes, stream);
        return v == 4 ? rows_typed<float, 4>(ZR_ARGS(float), stream) : rows_typed<float, 1>(ZR_ARGS(float), stream);
    }
    const int v = vec_width((const uint16_t*)Wt, (const uint16_t*)Wp, ld, N, 8);
    if (mode == ZR_DROP_N)
        return v >= 4 ? cols_typed<uint16_t, 4>(ZR_ARGS(uint16_t), workspace, workspace_bytes, stream)
                      : cols_typed<uint16_t, 1>(ZR_ARGS(uint16_t), workspace, workspace_bytes, stream);
    return v == 8 ? rows_typed<uint16_t, 8>(ZR_ARGS(uint16_t), stream)
         : v == 4 ? rows_typed<uint16_t, 4>(ZR_ARGS(uint16_t), stream)
                  : rows_typed<uint16_t, 1>(ZR_ARGS(uint16_t), stream);
#undef ZR_ARGS
}

int launch_priority_scores_static(const void* Wt, const void* Wp, int64_t ld, int K, int N, int mode,
                                  const float* prev_scores, const int32_t* prev_keep, int n_prev_keep,
                                  float* scores, int dtype, hipStream_t stream)
{
    if (priority_workspace_bytes(K, N, mode) > kStaticScratchBytes) return ZR_ERR_LIMIT;
    void* ws = nullptr;
    if (mode == ZR_DROP_N) {                    // row scores use no scratch
        const int st = static_scratch(&ws);
        if (st != ZR_OK) return st;
    }
    // every slot of the scratch that the finishing kernel reads is written by the summing
    // kernel of the same call first: nothing has to be cleared between calls
    return launch_priority_scores(Wt, Wp, ld, K, N, mode, prev_scores, prev_keep, n_prev_keep, scores, dtype,
                                  ws, ws ? kStaticScratchBytes : 0, stream);
}

size_t priority_static_scratch_bytes() { return kStaticScratchBytes; }

int launch_count_above(const float* scores, int n, float theta, int32_t* count, hipStream_t stream)
{
    hipLaunchKernelGGL(count_above_kernel, dim3(1), dim3(1024), 0, stream, scores, n, theta, count);
    return hip_status(hipGetLastError());
}

}  // namespace zr

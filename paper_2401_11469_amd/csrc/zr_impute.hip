// Stand-alone recovery/imputation pass (paper Sec. 3.1: the missing slices of a
// result are added back and filled by one of three policies: Zero, Same,
// Average).  HBM-bound: only the dropped slices are written (Zero), read and
// written (Same), or the kept ones read once and the dropped ones written
// (Average).  Kept slices are never touched.
#include "zr_common.h"

namespace zr {

namespace {

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<uint16_t> {   // bf16 storage
    static __device__ __forceinline__ float load(const uint16_t* p) { return bf16_bits_to_f32(*p); }
    static __device__ __forceinline__ void store(uint16_t* p, float v) { *p = (uint16_t)f32_to_bf16_bits(v); }
};

// true if p is in the ascending list keep[0..n_keep)
__device__ __forceinline__ bool is_kept(const int32_t* __restrict__ keep, int n_keep, int p)
{
    int lo = 0, hi = n_keep;          // first position with keep[pos] >= p
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (keep[mid] < p) lo = mid + 1; else hi = mid;
    }
    return lo < n_keep && keep[lo] == p;
}

constexpr int FILL_ROWS = 32;   // rows per workgroup of the column-fill kernel

// axis 1, ZERO / SAME: thread <-> one column, loops over a stripe of rows.
// Raw copies (bit-exact), so the element type is only a width.
template <typename T, bool SAME>
__global__ __launch_bounds__(256) void fill_cols_kernel(
    T* __restrict__ out, const T* __restrict__ prev, int64_t ld, int rows, int cols,
    const int32_t* __restrict__ keep, int n_keep)
{
    const int p = blockIdx.x * 256 + threadIdx.x;
    if (p >= cols) return;
    if (is_kept(keep, n_keep, p)) return;
    const int r0 = blockIdx.y * FILL_ROWS;
    const int r1 = min(rows, r0 + FILL_ROWS);
    for (int r = r0; r < r1; ++r) {
        const size_t off = (size_t)r * (size_t)ld + (size_t)p;
        out[off] = SAME ? prev[off] : T(0);
    }
}

// axis 0, ZERO / SAME: one workgroup per row; kept rows exit at once.
template <typename T, bool SAME>
__global__ __launch_bounds__(256) void fill_rows_kernel(
    T* __restrict__ out, const T* __restrict__ prev, int64_t ld, int rows, int cols,
    const int32_t* __restrict__ keep, int n_keep)
{
    const int r = blockIdx.x;
    if (is_kept(keep, n_keep, r)) return;
    T* o = out + (size_t)r * (size_t)ld;
    const T* q = SAME ? prev + (size_t)r * (size_t)ld : nullptr;
    for (int c = threadIdx.x; c < cols; c += 256) o[c] = SAME ? q[c] : T(0);
}

// axis 1, AVERAGE: one workgroup per row.  Sum of the kept columns in a fixed
// order (per-thread strided partial sums, then a fixed tree), so the result is
// deterministic; then every gap between kept columns receives the mean.
template <typename T>
__global__ __launch_bounds__(256) void average_cols_kernel(
    T* __restrict__ out, int64_t ld, int rows, int cols,
    const int32_t* __restrict__ keep, int n_keep)
{
    __shared__ float part[256];
    const int r = blockIdx.x;
    T* o = out + (size_t)r * (size_t)ld;
    float acc = 0.f;
    for (int q = threadIdx.x; q < n_keep; q += 256) acc += Elem<T>::load(o + clamp_idx(keep[q], cols));
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) part[threadIdx.x] += part[threadIdx.x + s];
        __syncthreads();
    }
    const float mean = part[0] / (float)n_keep;
    // gap q lies before kept column keep[q]; gap n_keep lies after the last one
    for (int q = threadIdx.x; q <= n_keep; q += 256) {
        const int lo = q == 0 ? 0 : clamp_idx(keep[q - 1], cols) + 1;
        const int hi = q == n_keep ? cols : clamp_idx(keep[q], cols);
        for (int p = lo; p < hi; ++p) Elem<T>::store(o + p, mean);
    }
}

// axis 0, AVERAGE: thread <-> one column; kept rows summed in ascending order.
template <typename T>
__global__ __launch_bounds__(256) void average_rows_kernel(
    T* __restrict__ out, int64_t ld, int rows, int cols,
    const int32_t* __restrict__ keep, int n_keep)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= cols) return;
    float acc = 0.f;
    for (int q = 0; q < n_keep; ++q)
        acc += Elem<T>::load(out + (size_t)clamp_idx(keep[q], rows) * (size_t)ld + c);
    const float mean = acc / (float)n_keep;
    for (int q = 0; q <= n_keep; ++q) {
        const int lo = q == 0 ? 0 : clamp_idx(keep[q - 1], rows) + 1;
        const int hi = q == n_keep ? rows : clamp_idx(keep[q], rows);
        for (int p = lo; p < hi; ++p) Elem<T>::store(out + (size_t)p * (size_t)ld + c, mean);
    }
}

// ---- Average from the per-tile sums of the product's epilogue ----------------
__global__ __launch_bounds__(256) void zero_f32_kernel(float* __restrict__ p, size_t count)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < count) p[i] = 0.f;
}

// mean over the kept slices, slots added in slot order; left in slot 0
__global__ __launch_bounds__(256) void mean_finish_kernel(float* __restrict__ partial, int slots, int len, int n_keep)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= len) return;
    float sum = 0.f;
    for (int s = 0; s < slots; ++s) sum += partial[(size_t)s * (size_t)len + i];
    partial[i] = sum / (float)n_keep;
}

// axis 1: dropped column p of row r receives mean[r]
template <typename T>
__global__ __launch_bounds__(256) void mean_fill_cols_kernel(
    T* __restrict__ out, int64_t ld, int rows, int cols, const int32_t* __restrict__ keep, int n_keep,
    const float* __restrict__ mean)
{
    const int p = blockIdx.x * 256 + threadIdx.x;
    if (p >= cols) return;
    if (is_kept(keep, n_keep, p)) return;
    const int r0 = blockIdx.y * FILL_ROWS;
    const int r1 = min(rows, r0 + FILL_ROWS);
    for (int r = r0; r < r1; ++r) Elem<T>::store(out + (size_t)r * (size_t)ld + (size_t)p, mean[r]);
}

// axis 0: dropped row r receives mean[c] in column c
template <typename T>
__global__ __launch_bounds__(256) void mean_fill_rows_kernel(
    T* __restrict__ out, int64_t ld, int rows, int cols, const int32_t* __restrict__ keep, int n_keep,
    const float* __restrict__ mean)
{
    const int r = blockIdx.x;
    if (is_kept(keep, n_keep, r)) return;
    T* o = out + (size_t)r * (size_t)ld;
    for (int c = threadIdx.x; c < cols; c += 256) Elem<T>::store(o + c, mean[c]);
}

template <typename T>
int mean_fill_typed(T* out, int64_t ld, int rows, int cols, int axis, const int32_t* keep, int n_keep,
                    float* partial, int slots, hipStream_t stream)
{
    const int len = axis == 1 ? rows : cols;
    hipLaunchKernelGGL(mean_finish_kernel, dim3((len + 255) / 256), dim3(256), 0, stream, partial, slots, len, n_keep);
    if (axis == 1) {
        dim3 grid((cols + 255) / 256, (rows + FILL_ROWS - 1) / FILL_ROWS);
        hipLaunchKernelGGL(mean_fill_cols_kernel<T>, grid, dim3(256), 0, stream, out, ld, rows, cols, keep, n_keep,
                           (const float*)partial);
    } else {
        hipLaunchKernelGGL(mean_fill_rows_kernel<T>, dim3(rows), dim3(256), 0, stream, out, ld, rows, cols, keep,
                           n_keep, (const float*)partial);
    }
    return hip_status(hipGetLastError());
}

template <typename T>
int impute_typed(T* out, int64_t ld, int rows, int cols, int axis, const int32_t* keep, int n_keep,
                 int policy, const T* prev, hipStream_t stream)
{
    const int n = axis == 0 ? rows : cols;
    if (n_keep == n) return ZR_OK;                       // nothing is missing
    if (policy == ZR_IMPUTE_SAME && prev == out) return ZR_OK;
    if (policy == ZR_IMPUTE_AVERAGE) {
        if (axis == 1)
            hipLaunchKernelGGL(average_cols_kernel<T>, dim3(rows), dim3(256), 0, stream,
                               out, ld, rows, cols, keep, n_keep);
        else
            hipLaunchKernelGGL(average_rows_kernel<T>, dim3((cols + 255) / 256), dim3(256), 0, stream,
                               out, ld, rows, cols, keep, n_keep);
    } else {
        const bool same = policy == ZR_IMPUTE_SAME;
        if (axis == 1) {
            dim3 grid((cols + 255) / 256, (rows + FILL_ROWS - 1) / FILL_ROWS);
            if (same) hipLaunchKernelGGL((fill_cols_kernel<T, true>), grid, dim3(256), 0, stream,
                                         out, prev, ld, rows, cols, keep, n_keep);
            else hipLaunchKernelGGL((fill_cols_kernel<T, false>), grid, dim3(256), 0, stream,
                                    out, prev, ld, rows, cols, keep, n_keep);
        } else {
            if (same) hipLaunchKernelGGL((fill_rows_kernel<T, true>), dim3(rows), dim3(256), 0, stream,
                                         out, prev, ld, rows, cols, keep, n_keep);
            else hipLaunchKernelGGL((fill_rows_kernel<T, false>), dim3(rows), dim3(256), 0, stream,
                                    out, prev, ld, rows, cols, keep, n_keep);
        }
    }
    return hip_status(hipGetLastError());
}

}  // namespace

int launch_zero_f32(float* p, size_t count, hipStream_t stream)
{
    if (count == 0) return ZR_OK;
    hipLaunchKernelGGL(zero_f32_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, stream, p, count);
    return hip_status(hipGetLastError());
}

int launch_mean_fill(void* out, int64_t ld, int rows, int cols, int axis, const int32_t* keep_idx, int n_keep,
                     float* partial, int slots, int dtype, hipStream_t stream)
{
    if (dtype == ZR_F32)
        return mean_fill_typed<float>((float*)out, ld, rows, cols, axis, keep_idx, n_keep, partial, slots, stream);
    return mean_fill_typed<uint16_t>((uint16_t*)out, ld, rows, cols, axis, keep_idx, n_keep, partial, slots, stream);
}

int launch_impute(void* out, int64_t ld, int rows, int cols, int axis,
                  const int32_t* keep_idx, int n_keep, int policy, const void* prev,
                  int dtype, hipStream_t stream)
{
    if (dtype == ZR_F32)
        return impute_typed<float>((float*)out, ld, rows, cols, axis, keep_idx, n_keep, policy,
                                   (const float*)prev, stream);
    return impute_typed<uint16_t>((uint16_t*)out, ld, rows, cols, axis, keep_idx, n_keep, policy,
                                  (const uint16_t*)prev, stream);
}

}  // namespace zr

// Extraction of the kept columns of an ACTIVATION tensor into a caller-provided
// workspace (the pruned input / pruned upstream gradient of paper Sec. 3.1: the
// kept columns side by side, in ascending index order).  Only activations are ever
// extracted; the weight shard is always gathered in flight by the GEMM loaders.
//
//   out[m, q] = in[m, S[q]]   for q <  n_keep
//   out[m, q] = +0            for n_keep <= q < width   (width = n_keep rounded up to 64)
//
// bf16 only (the fp32 path does not use it).  HBM-bound: reads M x n, writes
// M x width.  Main kernel: a workgroup brings a few whole rows into LDS with
// 16-byte loads (every byte of a touched line is fetched anyway: at the pruning
// ratios of interest the kept columns touch every 128-byte line), picks the kept
// elements out of LDS two at a time and stores dwords, 256 contiguous bytes per
// wavefront.  Fallback (rows that are not 16-byte aligned, or too long for LDS):
// one output dword is assembled from the two aligned input dwords that hold its
// elements with one byte permute.
#include "zr_common.h"

namespace zr {

namespace {

constexpr int CROWS = 8;   // rows per workgroup

__global__ __launch_bounds__(256) void compact_cols_kernel(
    const uint16_t* __restrict__ in, int64_t ld, int rows, int n,
    const int32_t* __restrict__ keep, int n_keep,
    uint16_t* __restrict__ out, int64_t ldo, int width)
{
    const int r0 = blockIdx.x * CROWS;
    const int nr = min(CROWS, rows - r0);
    for (int q = threadIdx.x; q < width / 2; q += 256) {
        const int c = 2 * q;
        const int a = clamp_idx(keep[min(c, n_keep - 1)], n);
        const int b = clamp_idx(keep[min(c + 1, n_keep - 1)], n);
        // byte selectors of v_perm: 0-3 from the first dword, 4-7 from the second, 0x0c -> 0x00
        const uint32_t lo = c < n_keep ? ((a & 1) ? 0x0302u : 0x0100u) : 0x0c0cu;
        const uint32_t hi = c + 1 < n_keep ? ((b & 1) ? 0x0706u : 0x0504u) : 0x0c0cu;
        const uint32_t sel = lo | (hi << 16);
        const uint16_t* p = in + (size_t)r0 * (size_t)ld;
        uint32_t* o = (uint32_t*)(out + (size_t)r0 * (size_t)ldo) + q;
        for (int r = 0; r < nr; ++r) {
            const uint32_t d0 = *(const uint32_t*)(p + (a & ~1));
            const uint32_t d1 = *(const uint32_t*)(p + (b & ~1));
            *o = __builtin_amdgcn_perm(d1, d0, sel);
            p += ld;
            o += ldo / 2;
        }
    }
}

// Rows staged through LDS.  RB rows of n elements each (n a multiple of 8, rows 16-byte
// aligned); thread t owns the output dwords t, t + 256, ... of every row of the group
// (their kept indices stay in registers for all RB rows).
template <int QMAX>
__global__ __launch_bounds__(256) void compact_rows_lds_kernel(
    const uint16_t* __restrict__ in, int64_t ld, int rows, int n,
    const int32_t* __restrict__ keep, int n_keep,
    uint16_t* __restrict__ out, int64_t ldo, int width, int rb)
{
    extern __shared__ __align__(16) uint16_t stage[];
    const int r0 = blockIdx.x * rb;
    const int nr = min(rb, rows - r0);
    const int chunks = n >> 3;
    // requests first: RB * n / 8 chunks of 16 bytes, consecutive threads on consecutive chunks
    const int total = nr * chunks;
    constexpr int LB = 8;                               // loads in flight per thread
    for (int u0 = threadIdx.x; u0 < total; u0 += 256 * LB) {
        uint4 v[LB];
#pragma unroll
        for (int k = 0; k < LB; ++k) {
            const int u = min(u0 + 256 * k, total - 1);
            const int r = u / chunks, c = u - r * chunks;
            v[k] = *(const uint4*)(in + (size_t)(r0 + r) * (size_t)ld + c * 8);
        }
#pragma unroll
        for (int k = 0; k < LB; ++k) {
            const int u = u0 + 256 * k;
            if (u < total) {
                const int r = u / chunks, c = u - r * chunks;
                *(uint4*)(stage + (size_t)r * n + c * 8) = v[k];
            }
        }
    }
    // thread t owns the output dwords (2 elements) t, t + 256, ... of every row: a wavefront
    // stores 256 contiguous bytes and its LDS reads are ~5 bytes apart from lane to lane
    // (8-byte stores with 4 reads per lane measured 15 % slower: more bank conflicts)
    int ia[QMAX], ib[QMAX];
    const int nq = width >> 1;
#pragma unroll
    for (int i = 0; i < QMAX; ++i) {
        const int c = 2 * (threadIdx.x + 256 * i);
        // beyond the kept count (zero padding): -1
        ia[i] = c < n_keep ? clamp_idx(keep[min(c, n_keep - 1)], n) : -1;
        ib[i] = c + 1 < n_keep ? clamp_idx(keep[min(c + 1, n_keep - 1)], n) : -1;
    }
    __syncthreads();
    for (int r = 0; r < nr; ++r) {
        const uint16_t* src = stage + (size_t)r * n;
        uint32_t* o = (uint32_t*)(out + (size_t)(r0 + r) * (size_t)ldo);
#pragma unroll
        for (int i = 0; i < QMAX; ++i) {
            const int q = threadIdx.x + 256 * i;
            if (q < nq) {
                const uint32_t lo = ia[i] >= 0 ? src[ia[i]] : 0u;
                const uint32_t hi = ib[i] >= 0 ? src[ib[i]] : 0u;
                o[q] = lo | (hi << 16);
            }
        }
    }
}

}  // namespace

// width: multiple of 64, <= ldo; ld, ldo even; in/out 4-byte aligned; n even.
int launch_compact_cols(const void* in, int64_t ld, int rows, int n, const int32_t* keep, int n_keep,
                        void* out, int64_t ldo, int width, hipStream_t stream)
{
    // LDS-staged rows when every row can be read in 16-byte chunks and a few rows fit
    const bool wide = (uintptr_t)in % 16 == 0 && ld % 8 == 0 && n % 8 == 0 && n <= 12288 && width <= 2 * 256 * 16;
    if (wide) {
        // rows per workgroup: few, so that thousands of workgroups even out over the CUs (2-4 measured
        // best; 8 rows lost 10-25 % to the last wave of workgroups); <= 24 KB of LDS
        const int rb = std::max(2, std::min(4, 8192 / n));
        const size_t smem = (size_t)rb * (size_t)n * 2;
        const int grid = (rows + rb - 1) / rb;
        const int qn = (width / 2 + 255) / 256;                         // output dwords per thread and row
#define ZR_COMPACT(Q)                                                                                         \
        hipLaunchKernelGGL(compact_rows_lds_kernel<Q>, dim3(grid), dim3(256), smem, stream, (const uint16_t*)in, ld, \
                           rows, n, keep, n_keep, (uint16_t*)out, ldo, width, rb)
        if (qn <= 2) ZR_COMPACT(2); else if (qn <= 4) ZR_COMPACT(4); else if (qn <= 8) ZR_COMPACT(8); else ZR_COMPACT(16);
#undef ZR_COMPACT
        return hip_status(hipGetLastError());
    }
    hipLaunchKernelGGL(compact_cols_kernel, dim3((rows + CROWS - 1) / CROWS), dim3(256), 0, stream,
                       (const uint16_t*)in, ld, rows, n, keep, n_keep, (uint16_t*)out, ldo, width);
    return hip_status(hipGetLastError());
}

}  // namespace zr

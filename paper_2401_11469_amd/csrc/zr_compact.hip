// Extraction of the kept columns of an ACTIVATION tensor into a caller-provided
// workspace (the paper's "pruned_input" / pruned upstream gradient, Sec. 3.1:
// the remaining columns concatenated in ascending index order).  Only
// activations are ever extracted; the weight shard is always gathered in
// flight by the GEMM loaders.
//
//   out[m, q] = in[m, S[q]]   for q <  n_keep
//   out[m, q] = +0            for n_keep <= q < width   (width = n_keep rounded up to 64)
//
// bf16 only (the fp32 path does not use it).  One output dword (two kept
// elements) is assembled from the two aligned input dwords that hold them with
// one byte permute, so all global accesses are 4 bytes wide and the stores
// are fully coalesced.  HBM-bound: reads M x n (touched lines), writes M x width.
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

}  // namespace

// width: multiple of 64, <= ldo; ld, ldo even; in/out 4-byte aligned; n even.
int launch_compact_cols(const void* in, int64_t ld, int rows, int n, const int32_t* keep, int n_keep,
                        void* out, int64_t ldo, int width, hipStream_t stream)
{
    hipLaunchKernelGGL(compact_cols_kernel, dim3((rows + CROWS - 1) / CROWS), dim3(256), 0, stream,
                       (const uint16_t*)in, ld, rows, n, keep, n_keep, (uint16_t*)out, ldo, width);
    return hip_status(hipGetLastError());
}

}  // namespace zr

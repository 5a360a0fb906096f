// Model of the main loop of the 256 x 256 x 64 bf16 GEMM tile in csrc/zr_gemm_fast.hip, for finding
// out which of its three streams overlap on gfx950.  Same grid (512 tiles of an 8192 x 4096 x 4096
// product), same workgroup -> tile map, same loads, barrier and instruction order; per 64-deep
// step and workgroup of 512 threads each stream can be switched on by itself:
//   1   64 KB of direct-to-LDS loads (8 per wavefront), requested at the top of the step
//   2   24 ds_read_b128 per wavefront (192 KB of fragment reads), read and used at once
//   4   32 MFMAs 32x32x16 per wavefront on register operands
//   8   the loads of (1) into registers instead (global_load_dwordx4)
//   64  the reads of (2) requested one MFMA step ahead, as the kernel does
//   256 with 64 and 4: the MFMAs take the fragments read as their operands, as the kernel does
//   512 with 4: twice as many MFMAs of half the size (16x16x32) instead of 32x32x16
// DEPTH = steps of loads in flight; SCHED = where in the step the loads are requested (see load_at).  Nothing is computed with the data; the output is time per
// step and the core clock (core ticks / 100 MHz wall ticks) seen by one workgroup.
// Build and run (stand-alone, not part of libzr):
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops loop_model.hip -o loop_model && ./loop_model
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstdint>
typedef __attribute__((address_space(3))) void* lds_void;
typedef const __attribute__((address_space(1))) void* glb_void;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Direct-to-LDS load written in assembly: the compiler's wait-count pass does not know of it, so
// every wait in the loop is the one written here (with the builtin it would make each fragment
// read wait for all loads in flight, because it cannot tell the two LDS stages apart).
__device__ __forceinline__ void dma16(const void* gptr, uint32_t* lds_uniform)
{
    const uint32_t l = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)lds_uniform);
    uint32_t saved_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0) : "v"(gptr), "s"(l) : "memory");
}

// SCHED 0: every wavefront requests its 8 loads at the top of the step.  SCHED 2: wavefronts 4-7
// (the SIMD mates of 0-3) request theirs two MFMA steps later.  SCHED 4: wavefronts 0-3 request
// all 16 loads of a SIMD pair.  SCHED 5: as 0, with the MFMAs issued at raised wave priority.
template <int MODE, int DEPTH = 1, int SCHED = 0>
__global__ __launch_bounds__(512) void mix(const uint16_t* A, const uint16_t* B, int ldk, int KT, int tiles_j, float* sink)
{
    extern __shared__ __align__(16) uint32_t smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per = gridDim.x / 8;
    const int t = (blockIdx.x % 8) * per + blockIdx.x / 8;
    const int GI = 4;
    const int grp_sz = GI * tiles_j;
    const int gidx = t / grp_sz, within = t - gidx * grp_sz;
    const int ti = gidx * GI + within % GI, tj = within / GI;
    const uint16_t* pa[4]; const uint16_t* pb[4];
    for (int q = 0; q < 4; ++q) {
        const int row = 8 * (wave + 8 * q) + (lane >> 3);
        pa[q] = A + (size_t)(ti * 256 + row) * ldk + (lane & 7) * 8;
        pb[q] = B + (size_t)(tj * 256 + row) * ldk + (lane & 7) * 8;
    }
    // zero the LDS once so that the fragment values are finite
    for (int i = tid; i < 32768; i += 512) smem[i] = 0x3e003d80u ^ ((uint32_t)i * 0x00010001u & 0x007f007fu);
    __syncthreads();
    const unsigned long long c0 = clock64(), w0 = wall_clock64();
    f32x16 acc[8];
    for (int c = 0; c < 8; ++c) for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
    f32x4 acc4[32];                 // the same 128 accumulator registers as 16 x 16 tiles (MODE & 512)
    for (int c = 0; c < 32; ++c) for (int r = 0; r < 4; ++r) acc4[c][r] = 0.f;
    bf16x8 fa, fb;
    for (int q = 0; q < 8; ++q) { fa[q] = (__bf16)(0.25f * ((lane + q) % 5)); fb[q] = (__bf16)(0.125f * ((lane * 3 + q) % 7)); }
    uint4 keep = make_uint4(0, 0, 0, 0);
    uint4 fr[2][6];
    for (int f = 0; f < 6; ++f) { fr[0][f] = make_uint4(0, 0, 0, 0); fr[1][f] = make_uint4(0, 0, 0, 0); }
    for (int kt = 0; kt < KT; ++kt) {
        uint32_t* wr = smem + ((kt + 1) & 1) * 16384;
        const uint32_t* rd = smem + (kt & 1) * 16384;
        auto load = [&](int q) {        // q = 0..7: four A instructions, then four B
            if (q < 4) dma16(pa[q] + kt * 64, wr + (wave + 8 * q) * 256);
            else dma16(pb[q - 4] + kt * 64, wr + 8192 + (wave + 8 * (q - 4)) * 256);
        };
        const int group = __builtin_amdgcn_readfirstlane(wave >> 2);
        if ((MODE & 1) && (SCHED == 0 || SCHED == 5)) {
#pragma unroll
            for (int q = 0; q < 8; ++q) load(q);
        }
        if ((MODE & 1) && SCHED == 4 && group == 0) {
            // wavefronts 0-3 request the whole tile (their own rows and their SIMD mates'), 4-7 nothing
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                load(q);
                if (q < 4) dma16(pa[q] + 32 * (size_t)ldk + kt * 64, wr + (wave + 4 + 8 * q) * 256);
                else dma16(pb[q - 4] + 32 * (size_t)ldk + kt * 64, wr + 8192 + (wave + 4 + 8 * (q - 4)) * 256);
            }
        }
        uint4 rg[8];
        if (MODE & 8) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                rg[q] = *(const uint4*)(pa[q] + kt * 64);
                rg[4 + q] = *(const uint4*)(pb[q] + kt * 64);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int step = 0; step < 4; ++step) {
            asm volatile("" ::: "memory");
            if ((MODE & 1) && SCHED == 2 && step == (group ? 2 : 0)) {
#pragma unroll
                for (int q = 0; q < 8; ++q) load(q);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (MODE & 64) {
                // fragments of the NEXT step requested before this step's MFMAs; the previous
                // request is consumed first (stands for the MFMAs needing their operands), or,
                // with 256, really is the MFMAs' operands (4 A and 2 B fragments, as in the kernel)
                const int cb = step & 1, nb = cb ^ 1;
                if (!(MODE & 256)) {
#pragma unroll
                    for (int f = 0; f < 6; ++f) { keep.x ^= fr[cb][f].x; keep.y ^= fr[cb][f].y; keep.z ^= fr[cb][f].z; keep.w ^= fr[cb][f].w; }
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int f = 0; f < 6; ++f) fr[nb][f] = *(const uint4*)(rd + ((((step + 1) & 3) * 6 + f) * 64 + lane) * 4);
                __builtin_amdgcn_sched_barrier(0);
            } else if (MODE & 2) {
                // 6 fragment reads per step: 16 B per lane, lanes on consecutive 16-byte slots (no bank conflicts)
#pragma unroll
                for (int f = 0; f < 6; ++f) {
                    const uint4 v = *(const uint4*)(rd + ((step * 6 + f) * 64 + lane) * 4);
                    keep.x ^= v.x; keep.y ^= v.y; keep.z ^= v.z; keep.w ^= v.w;
                }
            }
            if (MODE & 4) {
                if (SCHED == 5) __builtin_amdgcn_s_setprio(3);
                if (MODE & 512) {
                    // the same work as 16 MFMAs 16x16x32 (half the size each)
#pragma unroll
                    for (int c = 0; c < 16; ++c) {
                        const int t = (step & 1) * 16 + c;
                        if (MODE & 256) {
                            union { uint4 u; bf16x8 b; } xa, xb;
                            xa.u = fr[step & 1][c & 3]; xb.u = fr[step & 1][4 + ((c >> 2) & 1)];
                            acc4[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa.b, xb.b, acc4[t], 0, 0, 0);
                        } else {
                            acc4[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, acc4[t], 0, 0, 0);
                        }
                    }
                } else
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    if (MODE & 256) {
                        union { uint4 u; bf16x8 b; } xa, xb;
                        xa.u = fr[step & 1][c & 3]; xb.u = fr[step & 1][4 + (c >> 2)];
                        acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa.b, xb.b, acc[c], 0, 0, 0);
                    } else {
                        acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc[c], 0, 0, 0);
                    }
                }
                if (SCHED == 5) __builtin_amdgcn_s_setprio(0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (MODE & 8) {
#pragma unroll
            for (int q = 0; q < 8; ++q) { keep.x ^= rg[q].x; keep.y ^= rg[q].y; keep.z ^= rg[q].z; keep.w ^= rg[q].w; }
        }
        if (DEPTH == 1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (DEPTH == 2) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        if (DEPTH == 3) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        __builtin_amdgcn_s_barrier();
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    float s = 0.f;
    for (int c = 0; c < 8; ++c) for (int r = 0; r < 16; ++r) s += acc[c][r];
    for (int c = 0; c < 32; ++c) for (int r = 0; r < 4; ++r) s += acc4[c][r];
    if (s == 123.f || keep.x == 0x12345u) sink[blockIdx.x] = s + keep.y + keep.z + keep.w;
    if (blockIdx.x == 17 && tid == 0) {
        const unsigned long long c1 = clock64(), w1 = wall_clock64();
        ((unsigned long long*)(sink + 1024))[0] = c1 - c0;
        ((unsigned long long*)(sink + 1024))[1] = w1 - w0;
    }
}

// operands: small bf16 values of both signs (all-zero operands would make the MFMAs draw less power)
__global__ void fill(uint16_t* p, size_t n)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const uint32_t h = (uint32_t)(i * 2654435761u) >> 16;
        // sign, exponent 2^-4 .. 2^-1, 7 mantissa bits
        p[i] = (uint16_t)(((h & 1u) << 15) | ((123u + ((h >> 1) & 3u)) << 7) | ((h >> 3) & 127u));
    }
}

int main(int argc, char** argv)
{
    const int M = 8192, J = 4096, K = 4096;
    const int ld = K + 64;
    uint16_t *A, *B; float* sink;
    hipMalloc(&A, (size_t)M * ld * 2); hipMalloc(&B, (size_t)J * ld * 2); hipMalloc(&sink, 8192);
    hipLaunchKernelGGL(fill, dim3(1024), dim3(256), 0, 0, A, (size_t)M * ld);
    hipLaunchKernelGGL(fill, dim3(1024), dim3(256), 0, 0, B, (size_t)J * ld);
    const int tiles_i = M / 256, tiles_j = J / 256, KT = K / 64;
    const int grid = tiles_i * tiles_j;
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    auto run = [&](auto kern, const char* name) {
        hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 131072 + 2048);
        float best = 1e9f;
        for (int rep = 0; rep < 5; ++rep) {
            hipEventRecord(e0, 0);
            hipLaunchKernelGGL(kern, dim3(grid), dim3(512), 131072 + 2048, 0, A, B, ld, KT, tiles_j, sink);
            hipEventRecord(e1, 0); hipEventSynchronize(e1);
            float ms; hipEventElapsedTime(&ms, e0, e1); if (ms < best) best = ms;
        }
        unsigned long long cw[2];
        hipMemcpy(cw, sink + 1024, 16, hipMemcpyDeviceToHost);
        printf("%-28s %.1f us total, %.3f us per k-tile step; block 17: %llu core ticks / %llu wall ticks (100 MHz) = %.0f MHz\n", name, best * 1e3, best * 1e3 / (2.0 * KT),
               cw[0], cw[1], cw[1] ? (double)cw[0] / (double)cw[1] * 100.0 : 0.0);
        fflush(stdout);
    };
    run(mix<1>, "loads"); run(mix<1, 2>, "loads, 2 steps in flight"); run(mix<2>, "reads"); run(mix<4>, "mfma");
    run(mix<3>, "loads+reads"); run(mix<5>, "loads+mfma"); run(mix<5, 2>, "loads+mfma, 2 in flight");
    run(mix<8>, "register loads"); run(mix<12>, "register loads+mfma");
    run(mix<6>, "reads+mfma"); run(mix<64 + 4>, "reads ahead+mfma");
    run(mix<5, 1, 2>, "loads staggered+mfma");
    run(mix<7>, "ALL, reads used at once"); run(mix<64 + 5>, "ALL, reads ahead"); run(mix<64 + 5, 1, 2>, "ALL, reads ahead, loads staggered");
    run(mix<256 + 64 + 4>, "reads ahead feed the mfma"); run(mix<256 + 64 + 5>, "ALL, reads ahead feed the mfma"); run(mix<256 + 64 + 5, 1, 2>, "ALL, reads feed mfma, loads staggered");
    run(mix<5, 1, 4>, "loads by wavefronts 0-3 only+mfma"); run(mix<256 + 64 + 5, 1, 4>, "ALL, reads feed mfma, loads by wavefronts 0-3");
    run(mix<512 + 4>, "mfma 16x16x32"); run(mix<512 + 5>, "loads+mfma 16x16x32"); run(mix<512 + 256 + 64 + 5>, "ALL, reads feed mfma 16x16x32");
    run(mix<5, 1, 5>, "loads+mfma at raised priority"); run(mix<256 + 64 + 5, 1, 5>, "ALL, reads feed mfma, mfma at raised priority");
    hipError_t e = hipDeviceSynchronize();
    printf("status %s\n", hipGetErrorString(e));
    return e == hipSuccess ? 0 : 1;
}

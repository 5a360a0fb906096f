// Fast path of the gather-fused MFMA GEMM for bf16 tensors with 16-byte
// aligned rows (gfx950).  Same canonical product as the general kernel,
//     D[i, j] = sum_c A(i, c) * B(j, c),
// with large workgroup tiles (up to 256 x 256 x 64 on 8 wavefronts) because the
// L2 -> CU path sustains only ~40 B/clk/CU: a 256 x 256 tile needs 32 B/clk at
// full MFMA rate, a 128 x 128 one 64.
//
// How each kept-index gather of the resized products (paper Sec. 3.1) is fused
// into the load path, none of them through sub-dword global loads (those run
// at ~4 lanes/clk on this chip):
//   rows of a stored matrix (W[S,:], or any kept slice of a shard stored in the
//        layout that makes it rows) -> the row list only changes the row pointer
//        of the direct-to-LDS loads (loaders DmaP; DmaQM when the list runs
//        along the contraction axis and is walked tile by tile).
//   plain operands, and activations whose kept columns the caller's scratch
//        buffer already holds compacted -> direct-to-LDS loads (DmaP / DmaQ).
//   contiguous axis, non-contraction, no scratch -> the full-width span of the
//        tile's kept columns is fetched with 16-byte loads, memory rows are
//        interleaved in registers and only the kept columns' words are written to
//        LDS at their compacted positions (loader LdQG).
//   contiguous axis, contraction, no scratch -> each LDS word (two consecutive
//        kept indices of one row) is assembled from two aligned dword loads with
//        one byte permute (loader LdPG).
//   LdPV / LdQV: register-staged plain loaders for contraction extents that are
//        not a multiple of 64 when no operand supplies the zero tail.
// Epilogues: plain 16-byte stores; row scatter (kept rows to their original
// rows, dropped rows imputed); column scatter (the tile is laid out by original
// column in LDS, imputed value first, results on top, 16-byte stores).  Zero and
// Same imputation happen here; Average leaves per-tile sums for a fill pass.
#include <cstdio>
#include <cstdlib>
#include <type_traits>

#include "zr_common.h"
#include <cstring>

namespace zr {

namespace {

constexpr int BK = 64;           // contraction depth of one LDS tile (bf16 elements)
#ifndef ZR_BIG_WM
#define ZR_BIG_WM 2
#define ZR_BIG_WN 4
#endif

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Kernels whose two loaders are direct-to-LDS multiply with 16 x 16 x 32 MFMAs (twice as
// many instructions of half the size as 32 x 32 x 16): the loads of the next tile get
// into the instruction stream between them much better (measured on a model of the
// loop: 13 % less time per step with everything else equal).
#ifndef ZR_MFMA16
#define ZR_MFMA16 1
#endif
typedef uint16_t E;

// LDS tile layout of the register-staged loaders: 8 blocks (one per group of 8
// contraction indices); inside a block every tile row owns one 16-byte slot
// holding its 8 bf16 of that group, so an MFMA k-vector is one ds_read_b128.
// The LDS serves a 16-byte access 16 lanes at a time over 64 banks (256 bytes),
// so 16 lanes must hit 16 different slots modulo 16.  With i = 128 b + 8 a + m
// (m = i & 7) the row sits at slot 128 b + 16 m + ((a + 2 m) & 15): that holds
// both for 16 consecutive rows (fragment reads) and for rows 8 apart (writes of
// the loaders whose lanes hold 8 consecutive columns each).
template <int R> struct Tile {
    static constexpr int BW = R * 4 + 4;              // words per block (blocks 1 bank group out of phase)
    static constexpr int WORDS = 8 * BW;
    static __device__ __forceinline__ int slot(int i)
    {
        const int m = i & 7, a = (i >> 3) & 15;
        return (i & ~127) + 16 * m + ((a + 2 * m) & 15);
    }
};

typedef __attribute__((address_space(3))) void* lds_void;
typedef const __attribute__((address_space(1))) void* glb_void;
typedef short v4i16 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 as_frag(uint4 u)
{
    union { uint4 u; bf16x8 b; } x;
    x.u = u;
    return x.b;
}

// Fragment reader of the block/slot layout (register-staged loaders).
// w0: first tile row of this wavefront; t: 32-row sub-tile; step: 16 contraction
// indices; lanes 0-31 take the first 8 of them, lanes 32-63 the other 8.
template <int R> struct SlotReader {
    int off[4];     // word offset of this lane's row in each of the wavefront's 32-row sub-tiles
    __device__ __forceinline__ void setup(int w0, int lane)
    {
#pragma unroll
        for (int t = 0; t < 4; ++t)
            off[t] = Tile<R>::slot(min(w0 + t * 32 + (lane & 31), R - 1)) * 4 + (lane >> 5) * Tile<R>::BW;
    }
    __device__ __forceinline__ bf16x8 read(const uint32_t* stage, int t, int step) const
    {
        return as_frag(*(const uint4*)(stage + off[t] + 2 * step * Tile<R>::BW));
    }
};

struct FOp {
    const E* base;
    int64_t ld;
    const int32_t* map_s;   // row list (strided axis) or nullptr
    const int32_t* map_c;   // kept list on the contiguous axis or nullptr
    int n_s, n_c;           // memory extents
};

struct FArgs {
    FOp A, B;
    int I, J, C;
    E* out;
    int64_t ldo;
    int epilogue;
    const int32_t* keep;
    int out_full;
    const E* prev;          // Same imputation source (layout of out) or nullptr
    int accumulate;         // add the old contents of out (plain epilogue)
    float* avg_partial;     // Average imputation: per-tile sums of the stored results, or nullptr
    int avg_len;            // entries per slot of avg_partial
    int avg_slot_base;      // slot of this launch's first tile along the summed axis
    // Split contraction (products with too few tiles to fill the chip): phase 1 = every workgroup
    // multiplies one slice of the contraction of one tile and stores its fp32 accumulators to
    // `partial`; phase 2 = one workgroup per tile adds the slices in slice order and runs the
    // epilogue.  split <= 1: the ordinary single launch.
    float* partial;
    size_t partial_bytes;       // host side only: room at `partial`
    int split, phase, kt_per;   // kt_per: 64-deep contraction tiles per slice
    // sub-rectangle of D this launch covers, in elements (multiples of 256 except at
    // the far edges of D) and its tile grid
    int i_base, j_base, i_end, j_end;
    int tiles_i, tiles_j;
};

// fp32 -> bf16, round to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ E to_bf16(float f)
{
    union { __bf16 h; E u; } x;
    x.h = (__bf16)f;
    return x.u;
}

// rows[q] <- list[idx[q]] clamped into [0, n) (or idx[q] itself without a list); the
// loads are issued together under ONE uniform branch instead of one branch + wait each
template <int N>
__device__ __forceinline__ void lookup_rows(const int32_t* list, int n, const int (&idx)[N], int (&rows)[N])
{
    if (list) {
        int v[N];
#pragma unroll
        for (int q = 0; q < N; ++q) v[q] = list[idx[q]];
#pragma unroll
        for (int q = 0; q < N; ++q) rows[q] = clamp_idx(v[q], n);
    } else {
#pragma unroll
        for (int q = 0; q < N; ++q) rows[q] = idx[q];
    }
}

__device__ __forceinline__ uint4 zero4() { return make_uint4(0, 0, 0, 0); }
__device__ __forceinline__ uint4 sel4(bool ok, uint4 v)
{
    return make_uint4(ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u);
}

__device__ __forceinline__ int lower_bound_lds(const int* s, int n, int p)
{
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (s[mid] < p) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// Four memory rows (contraction indices c..c+3) x 8 consecutive columns ->
// for column m the two words (c,c+1) and (c+2,c+3).
__device__ __forceinline__ void interleave4x8(const uint4 r[4], uint2 w[8])
{
    const uint32_t a[4] = {r[0].x, r[0].y, r[0].z, r[0].w};
    const uint32_t b[4] = {r[1].x, r[1].y, r[1].z, r[1].w};
    const uint32_t c[4] = {r[2].x, r[2].y, r[2].z, r[2].w};
    const uint32_t d[4] = {r[3].x, r[3].y, r[3].z, r[3].w};
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        // v_perm byte selectors: 0-3 = second source, 4-7 = first source
        w[2 * t] = make_uint2(__builtin_amdgcn_perm(b[t], a[t], 0x05040100u),
                              __builtin_amdgcn_perm(d[t], c[t], 0x05040100u));
        w[2 * t + 1] = make_uint2(__builtin_amdgcn_perm(b[t], a[t], 0x07060302u),
                                  __builtin_amdgcn_perm(d[t], c[t], 0x07060302u));
    }
}

// ---------------------------------------------------------------------------
// Loaders.  Rows of the tile beyond the operand's extent are read from a
// clamped (valid) address and left as they are: they only feed rows / columns
// of D that the epilogue never stores.  The contraction tail (c >= C) is
// zeroed in every operand.  All fetches are branch-free so that the loads of
// tile k+1 stay in flight during the MFMAs of tile k.
// ---------------------------------------------------------------------------

// Contraction axis contiguous in memory, 16-byte loads, optional row list.
template <int R, int NT>
struct LdPV {
    static constexpr const char* NAME = "LdPV";
    static constexpr bool RING = false;
    typedef Tile<R> T;
    typedef SlotReader<R> Reader;
    static constexpr bool DMA = false;
    static constexpr int WORDS = Tile<R>::WORDS;
    static constexpr int N = R * 8 / NT;
    static constexpr bool NEEDS_IDX = false;
    const E* ptr[N];
    uint4 v[N];
    bool ok_;               // the fetched chunk lies inside the contraction range

    __device__ __forceinline__ void init(const FOp& op, int r0, int rlim, int tid, int*, int)
    {
        int idx[N], rows[N];
#pragma unroll
        for (int it = 0; it < N; ++it) idx[it] = min(r0 + ((tid + NT * it) >> 3), rlim - 1);
        lookup_rows<N>(op.map_s, op.n_s, idx, rows);
#pragma unroll
        for (int it = 0; it < N; ++it)
            ptr[it] = op.base + (size_t)rows[it] * (size_t)op.ld + ((tid + NT * it) & 7) * 8;
    }
    __device__ __forceinline__ void fetch(const FOp& op, int c0, int C, int tid)
    {
        const int c = c0 + (tid & 7) * 8;
        // a chunk is used if it starts inside the contraction range; it is always
        // whole inside the readable row (n_c is a multiple of 8, >= C)
        ok_ = c < C && c + 8 <= op.n_c;
        const int cc = ok_ ? c0 : -(tid & 7) * 8;    // past the tail: re-read the row start (zeroed in commit)
#pragma unroll
        for (int it = 0; it < N; ++it) v[it] = *(const uint4*)(ptr[it] + cc);
    }
    __device__ __forceinline__ void commit(const FOp&, uint32_t* lds, int tid)
    {
#pragma unroll
        for (int it = 0; it < N; ++it) {
            const int q = tid + NT * it;
            *(uint4*)(lds + (q & 7) * T::BW + T::slot(q >> 3) * 4) = sel4(ok_, v[it]);
        }
    }
};

// Contraction axis contiguous in memory with the kept list on it: word (row, cp)
// holds elements S[c0+2cp], S[c0+2cp+1] of the row, each cut out of its aligned
// dword with one byte permute.
template <int R, int NT>
struct LdPG {
    static constexpr const char* NAME = "LdPG";
    static constexpr bool RING = false;
    typedef Tile<R> T;
    typedef SlotReader<R> Reader;
    static constexpr bool DMA = false;
    static constexpr int WORDS = Tile<R>::WORDS;
    static constexpr int N = R * 32 / NT;
    static constexpr int RSTEP = NT / 32;
    static constexpr bool NEEDS_IDX = false;
    const E* rp;            // first row of this thread
    int64_t rstride;        // RSTEP rows, in elements
    int rmax;               // how many of the N rows exist (others are clamped)
    int sa, sb;             // source columns of the NEXT fetch (read one step ahead)
    uint32_t sel;
    uint32_t d0[N], d1[N];

    __device__ __forceinline__ void load_pair(const FOp& op, int c0, int C, int tid)
    {
        const int c = c0 + 2 * (tid & 31);
        sa = clamp_idx(op.map_c[min(c, C - 1)], op.n_c);
        sb = clamp_idx(op.map_c[min(c + 1, C - 1)], op.n_c);
    }
    __device__ __forceinline__ void init(const FOp& op, int r0, int rlim, int tid, int*, int C)
    {
        const int row = r0 + (tid >> 5);
        rp = op.base + (size_t)min(row, rlim - 1) * (size_t)op.ld;
        rstride = (int64_t)RSTEP * op.ld;
        rmax = row < rlim ? (rlim - 1 - row) / RSTEP + 1 : 0;
        load_pair(op, 0, C, tid);
    }
    __device__ __forceinline__ void fetch(const FOp& op, int c0, int C, int tid)
    {
        const int c = c0 + 2 * (tid & 31);
        const int a = sa, b = sb;
        // byte selectors of v_perm: 0-3 pick from d0, 4-7 from d1, 0x0c gives 0x00
        const uint32_t lo = c < C ? ((a & 1) ? 0x0302u : 0x0100u) : 0x0c0cu;
        const uint32_t hi = c + 1 < C ? ((b & 1) ? 0x0706u : 0x0504u) : 0x0c0cu;
        sel = lo | (hi << 16);
        const int oa = a & ~1, ob = b & ~1;
        const E* p = rp;
#pragma unroll
        for (int it = 0; it < N; ++it) {
            d0[it] = *(const uint32_t*)(p + oa);
            d1[it] = *(const uint32_t*)(p + ob);
            if (it + 1 < rmax) p += rstride;          // rows past the extent re-read the last one
        }
        load_pair(op, c0 + BK, C, tid);               // indices for the next tile
    }
    __device__ __forceinline__ void commit(const FOp&, uint32_t* lds, int tid)
    {
        const int cp = tid & 31;
        uint32_t* dst = lds + (cp >> 2) * T::BW + (cp & 3);
#pragma unroll
        for (int it = 0; it < N; ++it)
            dst[T::slot((tid >> 5) + RSTEP * it) * 4] = __builtin_amdgcn_perm(d1[it], d0[it], sel);
    }
};

// Contraction axis strided in memory: a unit is 4 memory rows (c..c+3) x 8
// consecutive columns, interleaved in registers; optional row list on c.
template <int R, int NT>
struct LdQV {
    static constexpr const char* NAME = "LdQV";
    static constexpr bool RING = false;
    typedef Tile<R> T;
    typedef SlotReader<R> Reader;
    static constexpr bool DMA = false;
    static constexpr int WORDS = Tile<R>::WORDS;
    static constexpr int UPR = R / 8;
    static constexpr int N = 16 * UPR / NT;
    static constexpr bool NEEDS_IDX = false;
    static_assert((16 * UPR) % NT == 0 && N >= 1, "unit count must divide over the threads");
    const E* colp[N];       // base + clamped column of the unit
    int rr[N][4];           // memory rows of the NEXT fetch
    uint4 v[N][4];
    int left_[N];           // contraction indices left from the unit's first row (<= 0: all past the tail)

    __device__ __forceinline__ void rows_for(const FOp& op, int c0, int C, int tid)
    {
        int idx[N * 4], rows[N * 4];
#pragma unroll
        for (int it = 0; it < N; ++it)
#pragma unroll
            for (int u = 0; u < 4; ++u) idx[it * 4 + u] = min(c0 + 4 * ((tid + NT * it) / UPR) + u, C - 1);
        lookup_rows<N * 4>(op.map_s, op.n_s, idx, rows);
#pragma unroll
        for (int it = 0; it < N; ++it)
#pragma unroll
            for (int u = 0; u < 4; ++u) rr[it][u] = rows[it * 4 + u];
    }
    __device__ __forceinline__ void init(const FOp& op, int r0, int rlim, int tid, int*, int C)
    {
#pragma unroll
        for (int it = 0; it < N; ++it) {
            // the readable row length n_c is a multiple of 8 (>= 8); columns past the
            // operand's extent are clamped into it and only feed discarded results
            const int j = min(r0 + ((tid + NT * it) % UPR) * 8, op.n_c - 8);
            colp[it] = op.base + j;
        }
        rows_for(op, 0, C, tid);
    }
    __device__ __forceinline__ void fetch(const FOp& op, int c0, int C, int tid)
    {
#pragma unroll
        for (int it = 0; it < N; ++it) {
            left_[it] = C - (c0 + 4 * ((tid + NT * it) / UPR));
#pragma unroll
            for (int u = 0; u < 4; ++u)
                v[it][u] = *(const uint4*)(colp[it] + (size_t)rr[it][u] * (size_t)op.ld);
        }
        rows_for(op, c0 + BK, C, tid);
    }
    __device__ __forceinline__ void commit(const FOp&, uint32_t* lds, int tid)
    {
#pragma unroll
        for (int it = 0; it < N; ++it) {
            const int q = tid + NT * it;
            const int kq = q / UPR, jc = q % UPR;
            uint2 w[8];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[it][u] = sel4(u < left_[it], v[it][u]);
            interleave4x8(v[it], w);
            uint32_t* dst = lds + (kq >> 1) * T::BW + (kq & 1) * 2 + (jc >> 4) * 512;
#pragma unroll
            for (int m = 0; m < 8; ++m) *(uint2*)(dst + (16 * m + ((jc + 2 * m) & 15)) * 4) = w[m];   // slot(8 jc + m)
        }
    }
};

// Contraction axis strided, kept list on the contiguous (non-contraction) axis:
// the tile's kept columns [r0, r0+cnt) of the list span the original columns
// [S[r0], S[r0+cnt-1]]; that span is fetched in aligned chunks of 8 columns
// (units of 4 memory rows x 8 columns) and only the kept columns are written
// to LDS, at their compacted rows.  Units beyond SLOTS*NT per tile (very sparse
// kept sets) are processed unpipelined in commit().
template <int R, int NT>
struct LdQG {
    static constexpr const char* NAME = "LdQG";
    static constexpr bool RING = false;
    typedef Tile<R> T;
    typedef SlotReader<R> Reader;
    static constexpr bool DMA = false;
    static constexpr int WORDS = Tile<R>::WORDS;
    static constexpr int SLOTS = 2;
    static constexpr bool NEEDS_IDX = true;
    const int* sidx;        // LDS copy of the tile's slice of the kept list
    int cnt, pa, nch, nunits, c0_, c_lim;
    const E* colp[SLOTS];
    uint32_t off[SLOTS][4]; // LDS word offsets (slot * 4) of the 8 columns, 16 bits each
    uint32_t meta[SLOTS];   // keep mask (bits 0-7) | kq << 8
    uint4 v[SLOTS][4];

    __device__ __forceinline__ void describe(const FOp& op, int q, const E*& cp, uint32_t o[4], uint32_t& mt)
    {
        const int kq = q / nch;
        const int p = pa + 8 * (q - kq * nch);
        int r = lower_bound_lds(sidx, cnt, p);
        uint32_t mask = 0;
        o[0] = o[1] = o[2] = o[3] = 0;
#pragma unroll
        for (int m = 0; m < 8; ++m) {
            const bool kept = r < cnt && sidx[r] == p + m;
            if (kept) {
                mask |= 1u << m;
                o[m >> 1] |= (uint32_t)(T::slot(r) * 4) << (16 * (m & 1));
                ++r;
            }
        }
        cp = op.base + p;
        mt = mask | ((uint32_t)kq << 8);
    }
    __device__ __forceinline__ void init(const FOp& op, int r0, int rlim, int tid, int* idx_lds, int C)
    {
        // idx_lds already holds clamp(S[r0 .. r0+cnt)) (filled by the kernel before init)
        sidx = idx_lds;
        c_lim = C;
        c0_ = 0;
        cnt = min(R, rlim - r0);
        pa = sidx[0] & ~7;
        nch = (sidx[cnt - 1] - pa) / 8 + 1;
        nunits = 16 * nch;
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const int q = tid + NT * s;
            if (q < nunits) {
                describe(op, q, colp[s], off[s], meta[s]);
            } else {
                colp[s] = op.base; meta[s] = 0;                      // nothing kept: no LDS write
                off[s][0] = off[s][1] = off[s][2] = off[s][3] = 0;
            }
        }
    }
    static __device__ __forceinline__ void load4(const FOp& op, const E* cp, int c, int C, uint4 r[4])
    {
#pragma unroll
        for (int u = 0; u < 4; ++u)
            r[u] = *(const uint4*)(cp + (size_t)min(c + u, C - 1) * (size_t)op.ld);
    }
    __device__ __forceinline__ void fetch(const FOp& op, int c0, int C, int)
    {
        c0_ = c0;
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) load4(op, colp[s], c0 + 4 * (int)(meta[s] >> 8), C, v[s]);
    }
    // left: contraction indices left from the unit's first row; rows past the tail become zero
    static __device__ __forceinline__ void scatter(uint32_t* lds, const uint4 r[4], const uint32_t o[4], uint32_t mt, int left)
    {
        uint2 w[8];
        uint4 z[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) z[u] = sel4(u < left, r[u]);
        interleave4x8(z, w);
        const int kq = (int)(mt >> 8);
        uint32_t* dst = lds + (kq >> 1) * T::BW + (kq & 1) * 2;
#pragma unroll
        for (int m = 0; m < 8; ++m)
            if (mt & (1u << m)) *(uint2*)(dst + ((o[m >> 1] >> (16 * (m & 1))) & 0xffffu)) = w[m];
    }
    __device__ __forceinline__ void commit(const FOp& op, uint32_t* lds, int tid)
    {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) scatter(lds, v[s], off[s], meta[s], c_lim - (c0_ + 4 * (int)(meta[s] >> 8)));
        for (int q = tid + NT * SLOTS; q < nunits; q += NT) {     // units that did not fit the slots
            const E* cp; uint32_t o[4], mt;
            describe(op, q, cp, o, mt);
            uint4 r[4];
            const int c = c0_ + 4 * (int)(mt >> 8);
            load4(op, cp, c, c_lim, r);
            scatter(lds, r, o, mt, c_lim - c);
        }
    }
};

// ---------------------------------------------------------------------------
// Direct-to-LDS loaders (global_load_lds_dwordx4): every lane names a 16-byte
// global chunk and the 64 chunks of a wavefront land back to back in 1 KB of
// LDS, so the layout is contiguous per instruction and bank conflicts are
// avoided by permuting WHICH chunk a lane fetches (XOR swizzles), never by
// padding.  No staging registers, no ds_write, and the L1 -> LDS path sustains
// ~56 B/clk/CU where loads into registers give ~32.
// A tile whose contraction extent is not a multiple of 64 re-reads valid data
// past the tail; the host only pairs such a tile with an operand that zeroes
// its own tail.
// ---------------------------------------------------------------------------

// Issued from inline assembly (m0 = LDS base of the instruction's 64 x 16 bytes; nothing else
// in these kernels reads m0).  With the builtin the compiler's wait-count pass counts the load
// against the LDS counter as well and then waits for ALL outstanding fragment reads (lgkmcnt(0))
// before every MFMA group; as it is, its lgkmcnt waits are exact and the vmcnt waits are the
// explicit ones of the pipeline.
#ifndef ZR_DMA_ASM
#define ZR_DMA_ASM 1
#endif
__device__ __forceinline__ void dma16(const void* gptr, uint32_t* lds_uniform)
{
#if ZR_DMA_ASM
    const uint32_t l = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)lds_uniform);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" :: "v"(gptr), "s"(l) : "memory");
#else
    __builtin_amdgcn_global_load_lds((glb_void)gptr, (lds_void)lds_uniform, 16, 0, 0);
#endif
}

// Contraction axis contiguous in memory (optional row list): LDS row i (128
// bytes) holds its 8 chunks at positions chunk ^ ((i >> 1) & 7), which spreads
// 16 consecutive rows of one chunk over all 64 banks.
template <int R, int NT>
struct DmaP {
    static constexpr const char* NAME = "DmaP";
    static constexpr bool RING = false;
    static constexpr bool DMA = true;
    static constexpr bool NEEDS_IDX = false;
    static constexpr int WORDS = R * 32;
    static constexpr int NW = NT / 64;
    static constexpr int N = R / 8 / NW;         // instructions per wavefront per tile
    const E* ptr[N];
    int chunk_;                                   // first contraction index of this lane's chunk

    struct Reader {
        int off, x;
        __device__ __forceinline__ void setup(int w0, int lane)
        {
            off = (w0 + (lane & 31)) * 32;
            x = (((lane >> 1) & 7) << 2) ^ ((lane >> 5) << 2);   // word offset of chunk grp ^ ((row >> 1) & 7)
        }
        __device__ __forceinline__ bf16x8 read(const uint32_t* stage, int t, int step) const
        {
            return as_frag(*(const uint4*)(stage + off + t * 1024 + (x ^ (step << 3))));
        }
        // 16 x 16 x 32 operands: lane = row (lane & 15) of sub-tile t, 8 contraction indices
        // from 8 (lane >> 4) of the 32-deep step: chunk 4 step + (lane >> 4)
        __device__ __forceinline__ void setup16(int w0, int lane)
        {
            off = (w0 + (lane & 15)) * 32;
            x = (((lane >> 1) & 7) << 2) ^ ((lane >> 4) << 2);
        }
        __device__ __forceinline__ bf16x8 read16(const uint32_t* stage, int t, int step) const
        {
            return as_frag(*(const uint4*)(stage + off + t * 512 + (x ^ (step << 4))));
        }
    };

    __device__ __forceinline__ void init(const FOp& op, int r0, int rlim, int tid, int*, int)
    {
        const int lane = tid & 63, wave = tid >> 6;
        // rows of an instruction: 8 (wave + NW q) + (lane >> 3); NW is even, so
        // (row >> 1) & 7 = 4 (wave & 1) + (lane >> 4) for every q
        static_assert(NW % 2 == 0, "the swizzle below assumes an even number of wavefronts");
        chunk_ = ((lane & 7) ^ (((lane >> 4) & 3) | ((wave & 1) << 2))) * 8;
        int idx[N], rows[N];
#pragma unroll
        for (int q = 0; q < N; ++q) idx[q] = min(r0 + 8 * (wave + NW * q) + (lane >> 3), rlim - 1);
        lookup_rows<N>(op.map_s, op.n_s, idx, rows);
#pragma unroll
        for (int q = 0; q < N; ++q) ptr[q] = op.base + (size_t)rows[q] * (size_t)op.ld;
    }
    __device__ __forceinline__ void issue(const FOp& op, uint32_t* stage, int c0, int C, int tid)
    {
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        const int c = min(c0 + chunk_, op.n_c - 8);              // the readable row length is a multiple of 8
#pragma unroll
        for (int q = 0; q < N; ++q) dma16(ptr[q] + c, stage + (wave + NW * q) * 256);
    }
    __device__ __forceinline__ void settle(const FOp&) {}
    // start the contraction at c0 instead of 0 (a slice of a split contraction): nothing to do,
    // issue() takes the offset as it comes
    __device__ __forceinline__ void seek(const FOp&, int, int, int) {}
};

// Contraction axis strided in memory (optional row list on it): LDS keeps the
// memory rows as they are (row c = R consecutive columns), with the 16-byte
// chunk index XORed by ZR_QSWZ * (c & 3); fragments are read with the transposing
// ds_read_tr16_b64, which hands a lane 4 consecutive c of ONE column out of a
// 4 (c) x 16 (columns) block read by its 16-lane group.  Two such groups (32
// lanes, 4 rows x 64 bytes) are served together; the rows are a multiple of
// 256 bytes apart, so the XOR has to move each of the 4 rows to its own
// 64-byte quarter of the 64 banks: factor 4 (a factor of 2 leaves rows 0/1 and
// 2/3 on the same banks; the conflict counter showed exactly that, 1 in 2).
// A tile width R that is not a power of two (192) keeps the LDS geometry of the
// next power of two RP: the lanes whose chunk lies beyond R are switched off,
// their LDS slots stay unwritten and are never read.
#ifndef ZR_QSWZ
#define ZR_QSWZ 4
#endif
// The 16 x 16 x 32 operand reads take 32 bytes from each of the rows 8 g .. 8 g + 3 per
// 16-lane group g; groups g and g + 1 are served together, so rows 8 apart must not
// share banks either: bit 3 of c moves the row by two more chunks (32 bytes).
#ifndef ZR_QSWZ8
#define ZR_QSWZ8 2
#endif
__device__ __forceinline__ constexpr int q_swizzle(int c) { return (ZR_QSWZ * (c & 3)) ^ (ZR_QSWZ8 * ((c >> 3) & 1)); }
// MAPPED: the memory rows go through a row list (W[S[c], :]).  A compile-time
// property, because a run-time "list or identity" choice inside the loop leaves a
// join whose register copies make the wavefront wait for every outstanding load,
// the tile's direct-to-LDS loads included, before its first MFMA.
template <int R, int NT, bool MAPPED>
struct DmaQT {
    static constexpr const char* NAME = MAPPED ? "DmaQM" : "DmaQ";
    static constexpr bool RING = false;
    static constexpr bool DMA = true;
    static constexpr bool NEEDS_IDX = false;
    static constexpr int RP = R <= 128 ? 128 : 256;
    static constexpr int WORDS = BK * RP / 2;
    static constexpr int NW = NT / 64;
    static constexpr int CPR = RP / 8;           // chunk slots per row
    static constexpr int RPI = 64 / CPR;         // rows per instruction
    static constexpr int N = CPR / NW;           // instructions per wavefront per tile
    static_assert(CPR % NW == 0 && N >= 1 && 64 % CPR == 0, "tile does not split over the wavefronts");
    static_assert(R % 64 == 0 && R <= RP && R > RP / 2, "unsupported tile width");
    const E* colp[N];
    int rr[N];                                    // memory row of the NEXT issue
    bool active_;                                 // this lane's chunk lies inside the tile

    struct Reader {
        int rowbase, coloff[4];
        __device__ __forceinline__ void setup(int w0, int lane)
        {
            const int t16 = lane & 15;
            rowbase = (8 * (lane >> 5) + (t16 >> 2)) * (RP / 2);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int col = w0 + t * 32 + 16 * ((lane >> 4) & 1) + 4 * (t16 & 3);
                coloff[t] = (((col >> 3) ^ q_swizzle(8 * (lane >> 5) + (t16 >> 2))) << 2) + ((col & 7) >> 1);
            }
        }
        __device__ __forceinline__ bf16x8 read(const uint32_t* stage, int t, int step) const
        {
            typedef __attribute__((address_space(3))) v4i16* lp;
            const uint32_t* p = stage + 16 * step * (RP / 2) + rowbase + coloff[t];
            union { v4i16 h[2]; bf16x8 b; } x;
            x.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)p);
            x.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)(p + 4 * (RP / 2)));
            return x.b;
        }
        // 16 x 16 x 32 operands: all four 16-lane groups read the sub-tile's 16 columns, group
        // g = lane >> 4 the contraction rows 8 g .. 8 g + 7 of the 32-deep step (two
        // transposing reads of 4 rows each).  Up to 8 sub-tiles per wavefront.
        int rowbase16, coloff16[8];
        __device__ __forceinline__ void setup16(int w0, int lane)
        {
            const int t16 = lane & 15;
            rowbase16 = (8 * (lane >> 4) + (t16 >> 2)) * (RP / 2);
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int col = w0 + t * 16 + 4 * (t16 & 3);
                coloff16[t] = (((col >> 3) ^ q_swizzle(8 * (lane >> 4) + (t16 >> 2))) << 2) + ((col & 7) >> 1);
            }
        }
        __device__ __forceinline__ bf16x8 read16(const uint32_t* stage, int t, int step) const
        {
            typedef __attribute__((address_space(3))) v4i16* lp;
            const uint32_t* p = stage + 32 * step * (RP / 2) + rowbase16 + coloff16[t];
            union { v4i16 h[2]; bf16x8 b; } x;
            x.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)p);
            x.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)(p + 4 * (RP / 2)));
            return x.b;
        }
    };

    __device__ __forceinline__ int tile_row(int q, int tid) const
    {
        return RPI * ((tid >> 6) + NW * q) + (tid & 63) / CPR;
    }
    __device__ __forceinline__ void rows_for(const FOp& op, int c0, int C, int tid)
    {
        int idx[N];
#pragma unroll
        for (int q = 0; q < N; ++q) idx[q] = min(c0 + tile_row(q, tid), C - 1);
        // with a list the entries are used as they arrive and clamped later, in settle()
#pragma unroll
        for (int q = 0; q < N; ++q) rr[q] = MAPPED ? op.map_s[idx[q]] : idx[q];
    }
    __device__ __forceinline__ void init(const FOp& op, int r0, int rlim, int tid, int*, int C)
    {
        // a lane's LDS slot is fixed; the XOR decides which chunk of the row it fetches.
        // The bits of tile_row(q) that enter the swizzle do not depend on q (instructions of
        // one wavefront are a multiple of 16 rows apart), so neither does the lane being
        // inside the tile
        static_assert(R == RP || (RPI * NW) % 16 == 0, "rows of successive instructions must agree modulo 16");
        active_ = (((tid & 63) % CPR) ^ q_swizzle(tile_row(0, tid))) * 8 < R;
#pragma unroll
        for (int q = 0; q < N; ++q) {
            const int chunk = ((tid & 63) % CPR) ^ q_swizzle(tile_row(q, tid));
            colp[q] = op.base + min(r0 + chunk * 8, op.n_c - 8);     // the readable row length is a multiple of 8
        }
        rows_for(op, 0, C, tid);
        settle(op);
    }
    __device__ __forceinline__ void issue(const FOp& op, uint32_t* stage, int c0, int C, int tid)
    {
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        if (R == RP || active_) {
#pragma unroll
            for (int q = 0; q < N; ++q)
                dma16(colp[q] + (size_t)rr[q] * (size_t)op.ld, stage + (wave + NW * q) * 256);
        }
        rows_for(op, c0 + BK, C, tid);
    }
    // start the contraction at c0 instead of 0 (a slice of a split contraction)
    __device__ __forceinline__ void seek(const FOp& op, int c0, int C, int tid)
    {
        rows_for(op, c0, C, tid);
        settle(op);
    }
    // Called after the MFMAs of the step: the row-list entries requested by issue() have
    // long arrived; clamping them here costs no wait and no time before the next issue.
    __device__ __forceinline__ void settle(const FOp& op)
    {
        if constexpr (MAPPED) {
#pragma unroll
            for (int q = 0; q < N; ++q) rr[q] = clamp_idx(rr[q], op.n_s);
        }
    }
};
template <int R, int NT> struct DmaQ : DmaQT<R, NT, false> {};
template <int R, int NT> struct DmaQM : DmaQT<R, NT, true> {};


// ---------------------------------------------------------------------------
// Ring pipeline (direct-to-LDS loaders only).  The contraction runs in stages of
// 32; four stages of LDS form a ring: while stage s is multiplied, the fragments
// of stage s+1 are already being read (it became visible at the previous
// barrier), stage s+2 is landing and stage s+3 is being requested.  What this
// buys over two 64-deep stages, all of it measured on a model of the loop first:
//  * every load is requested three stages (> 1 us) before it is needed, so the
//    requests can be spread over the step, ONE between two MFMAs at a time (a
//    wavefront stalls at a vector-memory instruction until the address unit takes
//    it, and the MFMAs queued behind it wait too), and nobody waits for vmcnt(0);
//  * one fragment read between two MFMAs instead of bursts in front of a group;
//  * the first fragments of a step are read before the barrier that ends the
//    previous one, so no MFMA waits for an LDS round trip after a barrier;
//  * the loads are issued from inline assembly: the compiler's wait-count pass
//    does not know of them, so its lgkmcnt waits stay exact (with the builtin it
//    waited for ALL outstanding LDS reads before every MFMA group) and the vmcnt
//    waits are the ones written here; the LDS address of a load is a scalar and
//    the global pointers advance by additions (the 64-deep loop spent ~40 vector
//    ALU instructions per step on addresses, between the barrier and its first MFMA).
// ---------------------------------------------------------------------------
constexpr int RK = 32;
#ifndef ZR_RING_PEEL
#define ZR_RING_PEEL 1
#endif
#ifndef ZR_RING_LSLOT
#define ZR_RING_LSLOT 2
#endif
#ifndef ZR_RING_ADIST
#define ZR_RING_ADIST 2
#endif
#ifndef ZR_RING_LEARLY
#define ZR_RING_LEARLY 0
#endif

__device__ __forceinline__ void dma16_ring(const void* gptr, uint32_t lds_byte_addr_uniform)
{
    // m0 = LDS base of the 64 x 16 bytes this instruction writes; no restore: nothing else
    // in these kernels reads m0
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :: "v"(gptr), "s"(lds_byte_addr_uniform) : "memory");
}

// Contraction axis contiguous (optional row list on the other axis): an LDS row is the
// 64 bytes (4 chunks) of one tile row; chunk c of row i sits at position c ^ ((i >> 1) & 3).
// Measured with a ds_read_b128 loop over the candidate swizzles: this one (and its like with
// bit 1 of the row in it) reads at the rate of a linear pattern, 256 bytes per clock;
// c ^ ((i >> 2) & 3), which also gives 16 consecutive rows 16 different bank groups, is 58 %
// slower and showed in the counters as one conflict cycle in two.  One instruction brings 16 rows.
template <int R, int NT>
struct RingP {
    static constexpr const char* NAME = "RingP";
    static constexpr bool RING = true, DMA = true, NEEDS_IDX = false, MAPPED = false;
    static constexpr int WORDS = R * 16;
    static constexpr int NW = NT / 64;
    static constexpr int NINST = R / 16;                    // instructions per stage
    // whole instructions per wavefront, or (192 rows on 8 wavefronts) half of the wavefronts
    // with one more than the others
    static constexpr bool FITS = NINST % NW == 0 || NINST % NW == NW / 2;
    static constexpr int NI = (NINST + NW - 1) / NW;
    static constexpr int SHORT = NINST % NW == 0 ? 0 : 1;   // instructions the higher wavefronts leave out
    const E* ptr[NI];
    int chunk_;
    uint32_t wave_;

    struct Reader {
        int off;
        __device__ __forceinline__ void setup16(int w0, int lane)
        {
            const int r = lane & 15;
            off = (w0 + r) * 16 + ((((lane >> 4) ^ (r >> 1)) & 3) << 2);
        }
        __device__ __forceinline__ bf16x8 read16(const uint32_t* stage, int t, int) const
        {
            return as_frag(*(const uint4*)(stage + off + t * 256));
        }
    };

    // how many of its NI instructions this wavefront issues per stage
    __device__ __forceinline__ int count() const { return SHORT && wave_ >= (uint32_t)(NINST % NW) ? NI - 1 : NI; }

    __device__ __forceinline__ void init(const FOp& op, int r0, int rlim, int tid, const int*, int)
    {
        const int lane = tid & 63;
        wave_ = __builtin_amdgcn_readfirstlane(tid >> 6);
        chunk_ = ((lane & 3) ^ ((lane >> 3) & 3)) * 8;         // row of the lane = lane >> 2
        int idx[NI], rows[NI];
#pragma unroll
        for (int q = 0; q < NI; ++q) idx[q] = min(r0 + 16 * ((int)wave_ + NW * q) + (lane >> 2), rlim - 1);
        lookup_rows<NI>(op.map_s, op.n_s, idx, rows);
#pragma unroll
        for (int q = 0; q < NI; ++q) ptr[q] = op.base + (size_t)rows[q] * (size_t)op.ld;
    }
    __device__ __forceinline__ void issue(const FOp& op, int q, uint32_t lds_bytes, int s, int)
    {
        if (SHORT && q == NI - 1 && wave_ >= (uint32_t)(NINST % NW)) return;      // uniform
        const int c = min(s * RK + chunk_, op.n_c - 8);          // the readable row length is a multiple of 8
        dma16_ring(ptr[q] + c, lds_bytes + (wave_ + NW * q) * 1024u);
    }
};

// Contraction axis strided (optional row list on it, kept in LDS): the LDS stage keeps the 32
// memory rows as they are, chunk index swizzled as in the 64-deep loader; fragments through
// the transposing reads.
template <int R, int NT, bool MAPPED_>
struct RingQT {
    static constexpr const char* NAME = MAPPED_ ? "RingQM" : "RingQ";
    static constexpr bool RING = true, DMA = true, NEEDS_IDX = false, MAPPED = MAPPED_;
    static constexpr int RP = R <= 128 ? 128 : 256;
    static constexpr int WORDS = RK * RP / 2;
    static constexpr int NW = NT / 64;
    static constexpr int CPR = RP / 8;           // chunk slots per row
    static constexpr int RPI = 64 / CPR;         // rows per instruction
    static constexpr bool FITS = (RK / RPI) % NW == 0 && R % 64 == 0 && R > RP / 2 && (RPI * NW) % 16 == 0;
    static constexpr int NI = FITS ? RK / RPI / NW : 1;
    static constexpr int SHORT = 0;
    __device__ __forceinline__ int count() const { return NI; }
    const E* colp;
    int row_[NI];                                 // row of the stage this lane fetches, per instruction
    bool active_;
    uint32_t wave_;
    const int* list_;                             // LDS copy of the row list (MAPPED)

    struct Reader {
        int rowbase16, coloff16[8];
        __device__ __forceinline__ void setup16(int w0, int lane)
        {
            const int t16 = lane & 15;
            rowbase16 = (8 * (lane >> 4) + (t16 >> 2)) * (RP / 2);
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int col = w0 + t * 16 + 4 * (t16 & 3);
                coloff16[t] = (((col >> 3) ^ q_swizzle(8 * (lane >> 4) + (t16 >> 2))) << 2) + ((col & 7) >> 1);
            }
        }
        __device__ __forceinline__ bf16x8 read16(const uint32_t* stage, int t, int) const
        {
            typedef __attribute__((address_space(3))) v4i16* lp;
            const uint32_t* p = stage + rowbase16 + coloff16[t];
            union { v4i16 h[2]; bf16x8 b; } x;
            x.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)p);
            x.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)(p + 4 * (RP / 2)));
            return x.b;
        }
    };

    __device__ __forceinline__ void init(const FOp& op, int r0, int, int tid, const int* list_lds, int)
    {
        const int lane = tid & 63;
        wave_ = __builtin_amdgcn_readfirstlane(tid >> 6);
        list_ = list_lds;
        // the swizzle bits of a lane's row do not depend on the instruction (rows of successive
        // instructions of a wavefront are 16 apart), so neither does the chunk it fetches
        static_assert(!FITS || (RPI * NW) % 16 == 0, "rows of successive instructions must agree modulo 16");
#pragma unroll
        for (int q = 0; q < NI; ++q) row_[q] = RPI * ((int)wave_ + NW * q) + lane / CPR;
        const int chunk = (lane % CPR) ^ q_swizzle(row_[0]);
        active_ = chunk * 8 < R;
        colp = op.base + min(r0 + chunk * 8, op.n_c - 8);        // the readable row length is a multiple of 8
    }
    __device__ __forceinline__ void issue(const FOp& op, int q, uint32_t lds_bytes, int s, int C)
    {
        int row = min(s * RK + row_[q], C - 1);
        if constexpr (MAPPED_) row = list_[row];                  // clamped when it was copied to LDS
        if (R == RP || active_) dma16_ring(colp + (size_t)row * (size_t)op.ld, lds_bytes + (wave_ + NW * q) * 1024u);
    }
};
template <int R, int NT> struct RingQ : RingQT<R, NT, false> {};
template <int R, int NT> struct RingQM : RingQT<R, NT, true> {};

// the ring loader that replaces a 64-deep direct-to-LDS loader
template <template <int, int> class L> struct RingOf { static constexpr bool has = false; };
template <> struct RingOf<DmaP> { static constexpr bool has = true; template <int R, int NT> using type = RingP<R, NT>; };
template <> struct RingOf<DmaQ> { static constexpr bool has = true; template <int R, int NT> using type = RingQ<R, NT>; };
template <> struct RingOf<DmaQM> { static constexpr bool has = true; template <int R, int NT> using type = RingQM<R, NT>; };

// which memory instruction, if any, follows MFMA b of row group gi of a step
__device__ __forceinline__ constexpr int ring_b_read(int gi, int b, int TM, int TN)
{
    if (TN <= TM - 1) return (b == 1 && gi >= TM - 1 - TN && gi < TM - 1) ? gi - (TM - 1 - TN) : -1;
    // two per group from the first group on
    if (b == 1) return 2 * gi < TN ? 2 * gi : -1;
    if (b == 3) return 2 * gi + 1 < TN ? 2 * gi + 1 : -1;
    return -1;
}
__device__ __forceinline__ constexpr int ring_load(int gi, int b, int TM, int NLW)
{
    if (b != ZR_RING_LSLOT) return -1;
    for (int j = 0; j < NLW; ++j)
        if ((ZR_RING_LEARLY ? j : (j * TM) / NLW) == gi) return j;
    return -1;
}

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// The whole contraction of one tile.  KT2 (even) stages of 32.
template <class LA, class LB, int TM, int TN>
__device__ __forceinline__ void ring_main(LA& la, LB& lb, const typename LA::Reader& ra, const typename LB::Reader& rb,
                                          const FArgs& g, uint32_t* smem, int s0, int KT2, f32x4 (&acc)[TM][TN])
{
    // s0: first stage (of 32) of this workgroup's share of the contraction; LDS slots go by the
    // stage's number within the share, addresses by its absolute number
    constexpr int A_WORDS = LA::WORDS, STAGE_WORDS = LA::WORDS + LB::WORDS;
    constexpr int NA = LA::NI, NLW = LA::NI + LB::NI;
    constexpr int RA = TM % 4 == 0 ? 4 : 3;                 // depth of the ring of A fragments
    static_assert(TM % RA == 0 && TM >= 4 && TN >= 4 && NLW <= TM, "schedule below does not fit this wavefront tile");
    static_assert(TN <= TM - 1 || 2 * (TM - 1) >= TN, "not enough slots for the B fragments");
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)smem);
    auto load = [&](int s, int j) {
        const uint32_t base = lds0 + (uint32_t)(s & 3) * (uint32_t)(STAGE_WORDS * 4);
        if (j < NA) la.issue(g.A, j, base, s0 + s, g.C);
        else lb.issue(g.B, j - NA, base + A_WORDS * 4, s0 + s, g.C);
    };
    for (int st = 0; st < 3; ++st) {
        if (st < KT2) {
#pragma unroll
            for (int j = 0; j < NLW; ++j) load(st, j);
        }
    }
    // a wavefront waits until at most ITS requests of one stage are outstanding (a loader whose
    // instructions do not divide over the wavefronts leaves some with one fewer)
    const int mine = la.count() + lb.count();
    auto wait_one_stage = [&] {
        if constexpr (LA::SHORT + LB::SHORT == 0) wait_vmcnt<NLW>();
        else if (mine == NLW) wait_vmcnt<NLW>();
        else if (mine == NLW - 1) wait_vmcnt<NLW - 1>();
        else wait_vmcnt<(NLW >= 2 ? NLW - 2 : 0)>();
    };
    if (KT2 > 2) wait_one_stage(); else wait_vmcnt<0>();      // stages 0 and 1 have landed
    __builtin_amdgcn_s_barrier();

    bf16x8 bfr[2][TN], afr[RA];
#pragma unroll
    for (int b = 0; b < TN; ++b) bfr[0][b] = rb.read16(smem + A_WORDS, b, 0);
    afr[0] = ra.read16(smem, 0, 0);
    afr[1] = ra.read16(smem, 1, 0);
    if (ZR_RING_ADIST == 3 && RA == 4) afr[2] = ra.read16(smem, 2, 0);

    // steady: the step is known to have a stage s + 3 to request (no branches around the loads)
    auto step = [&](int s, auto parity, auto steady) {
        constexpr int P = decltype(parity)::value;
        constexpr bool STEADY = decltype(steady)::value;
        const uint32_t* rd = smem + (s & 3) * STAGE_WORDS;
        const uint32_t* nx = smem + ((s + 1) & 3) * STAGE_WORDS;
        const bool more = STEADY || s + 3 < KT2;
#pragma unroll
        for (int gi = 0; gi < TM; ++gi) {
#pragma unroll
            for (int b = 0; b < TN; ++b) {
                acc[gi][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afr[gi % RA], bfr[P][b], acc[gi][b], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (b == 0) {
                    // row group gi + AD of this stage, or of the next one (visible since the last
                    // barrier; after the last stage this reads stale LDS that nothing uses)
                    constexpr int AD = (ZR_RING_ADIST == 3 && RA == 4) ? 3 : 2;
                    afr[(gi + AD) % RA] = gi + AD < TM ? ra.read16(rd, gi + AD, 0) : ra.read16(nx, gi + AD - TM, 0);
                }
                const int jb = ring_b_read(gi, b, TM, TN);
                if (jb >= 0) bfr[P ^ 1][jb] = rb.read16(nx + A_WORDS, jb, 0);
                const int jl = ring_load(gi, b, TM, NLW);
                if (jl >= 0 && more) load(s + 3, jl);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // stage s + 2 (requested during step s - 1) has landed when at most this step's requests are out
        if (more) wait_one_stage(); else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
    };
    int s = 0;
#if ZR_RING_PEEL
    for (; s + 4 < KT2; s += 2) {
        step(s, std::integral_constant<int, 0>(), std::true_type());
        step(s + 1, std::integral_constant<int, 1>(), std::true_type());
    }
#endif
    for (; s < KT2; s += 2) {           // the last stages: nothing left to request
        step(s, std::integral_constant<int, 0>(), std::false_type());
        step(s + 1, std::integral_constant<int, 1>(), std::false_type());
    }
}

// LDS of a workgroup: the stages (two of 64 or, for the ring loaders, four of 32) or the C tile
// of the epilogue, whichever is larger; then one kept-list entry per tile row and column; then,
// for a ring loader with a row list on the contraction axis, that list.
template <class LA, class LB> constexpr bool ring_mapped() { return false; }
template <int AW, int BW_, int BM, int BN, bool RING = false>
constexpr int fast_smem_bytes()
{
    constexpr int stage_bytes = (RING ? 4 : 2) * (AW + BW_) * 4;
    constexpr int c_bytes = BM * (BN + 8) * 2;
    return (stage_bytes > c_bytes ? stage_bytes : c_bytes) + (BM + BN) * 4;
}
// entries of the LDS copy of the row list (what is left of 160 KB, or of 80 KB for the tiles
// that run two to a compute unit)
template <int BM, int BN> constexpr int ring_list_max() { return BM * BN > 128 * 128 ? 6144 : 3072; }

// One iteration of the contraction pipeline.  `rd` (the stage being multiplied)
// and `wr` (the stage being filled) never overlap; declaring that lets the
// compiler keep the direct-to-LDS loads in flight across the fragment reads
// instead of waiting for them before the first ds_read.
template <class LA, class LB, int TM, int TN, class ACC>
__device__ __forceinline__ void pipeline_step(
    LA& la, LB& lb, const typename LA::Reader& ra, const typename LB::Reader& rb,
    const FArgs& g, const uint32_t* __restrict__ rd, uint32_t* __restrict__ wr,
    int c_next, bool more, int tid, ACC (&acc)[TM][TN])
{
    constexpr int A_WORDS = LA::WORDS;
    constexpr bool M16 = sizeof(ACC) == 16;
    if (more) {
        if constexpr (LA::DMA) la.issue(g.A, wr, c_next, g.C, tid); else la.fetch(g.A, c_next, g.C, tid);
        if constexpr (LB::DMA) lb.issue(g.B, wr + A_WORDS, c_next, g.C, tid); else lb.fetch(g.B, c_next, g.C, tid);
    }
    if constexpr (M16) {
        // Two 32-deep steps of TM groups (one A fragment against the step's TN B fragments).
        // The A fragments run through a ring of three, requested two groups ahead; the B
        // fragments of the second step are requested during the first step's last groups.
        // So after the first group of a tile no MFMA waits for an LDS round trip, with 44
        // fragment registers instead of the 96 that two whole steps would take.
        constexpr int STEPS = BK / 32, G = STEPS * TM;
        static_assert(TM >= 3, "the ring below is three deep");
        bf16x8 bfr[2][TN], afr[3];
#pragma unroll
        for (int b = 0; b < TN; ++b) bfr[0][b] = rb.read16(rd + A_WORDS, b, 0);
        afr[0] = ra.read16(rd, 0, 0);
        afr[1] = ra.read16(rd, 1, 0);
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
            const int step = gi / TM;
            if (gi + 2 < G) afr[(gi + 2) % 3] = ra.read16(rd, (gi + 2) % TM, (gi + 2) / TM);
            if (step + 1 < STEPS && gi % TM == TM - 3) {
#pragma unroll
                for (int b = 0; b < TN; ++b) bfr[(step + 1) & 1][b] = rb.read16(rd + A_WORDS, b, step + 1);
            }
            __builtin_amdgcn_sched_barrier(0);       // the requests stay above the MFMAs
#pragma unroll
            for (int b = 0; b < TN; ++b)
                acc[gi % TM][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afr[gi % 3], bfr[step & 1][b], acc[gi % TM][b], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    } else if constexpr (LA::DMA && LB::DMA) {
        // No staging registers are live here, so there is room to request the
        // fragments of step s+1 before the MFMAs of step s are issued: the LDS
        // latency hides behind this wavefront's own MFMAs.
        bf16x8 af[2][TM], bf[2][TN];
#pragma unroll
        for (int a = 0; a < TM; ++a) af[0][a] = ra.read(rd, a, 0);
#pragma unroll
        for (int b = 0; b < TN; ++b) bf[0][b] = rb.read(rd + A_WORDS, b, 0);
#pragma unroll
        for (int step = 0; step < BK / 16; ++step) {
            const int cb = step & 1, nb = cb ^ 1;
            if (step + 1 < BK / 16) {
#pragma unroll
                for (int a = 0; a < TM; ++a) af[nb][a] = ra.read(rd, a, step + 1);
#pragma unroll
                for (int b = 0; b < TN; ++b) bf[nb][b] = rb.read(rd + A_WORDS, b, step + 1);
            }
            __builtin_amdgcn_sched_barrier(0);       // keep the prefetch above the MFMAs
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[cb][a], bf[cb][b], acc[a][b], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
#pragma unroll
        for (int step = 0; step < BK / 16; ++step) {
            bf16x8 af[TM], bf[TN];
#pragma unroll
            for (int a = 0; a < TM; ++a) af[a] = ra.read(rd, a, step);
#pragma unroll
            for (int b = 0; b < TN; ++b) bf[b] = rb.read(rd + A_WORDS, b, step);
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bf[b], acc[a][b], 0, 0, 0);
        }
    }
    if (more) {
        if constexpr (LA::DMA) la.settle(g.A);
        if constexpr (LB::DMA) lb.settle(g.B);
        if constexpr (!LA::DMA) la.commit(g.A, wr, tid);
        if constexpr (!LB::DMA) lb.commit(g.B, wr + A_WORDS, tid);
        // direct-to-LDS loads are only tracked by the vector-memory counter: vmcnt(0)
        if constexpr (LA::DMA || LB::DMA) __builtin_amdgcn_s_waitcnt(0x0f70);
    }
}

// PHASE: 0 = the whole product in one launch; 1 / 2 = the two launches of a split contraction
// (instantiated for the 128 x 128 direct-to-LDS tiles only: separate kernels, so that the
// ordinary one keeps its register allocation).
template <template <int, int> class LA_, template <int, int> class LB_, int BM, int BN, int WM, int WN, int PHASE = 0>
__global__ __launch_bounds__(64 * WM * WN) void fast_kernel(const FArgs g)
{
    constexpr int NT = 64 * WM * WN;
    typedef LA_<BM, NT> LA;
    typedef LB_<BN, NT> LB;
    // (not where both operands come through the transposing reads on a tile larger than
    // 128 x 128: measured 1-2 % slower there, 10 % faster on the 128 x 128 tiles)
    constexpr bool RING = LA::RING;
    static_assert(LA::RING == LB::RING, "ring loaders come in pairs");
    constexpr bool both_transposed = LA::NAME[3] == 'Q' && LB::NAME[3] == 'Q';
    constexpr bool M16 = RING || (ZR_MFMA16 && LA::DMA && LB::DMA && !(both_transposed && BM * BN > 128 * 128));
    constexpr int MT = M16 ? 16 : 32;                  // rows and columns of one MFMA result tile
    constexpr int AR = M16 ? 4 : 16;                   // accumulator registers per tile and lane
    constexpr int TM = BM / (MT * WM), TN = BN / (MT * WN);
    typedef typename std::conditional<M16, f32x4, f32x16>::type ACC;
    constexpr int A_WORDS = LA::WORDS;
    constexpr int B_WORDS = LB::WORDS;
    constexpr int STAGE_WORDS = A_WORDS + B_WORDS;
    constexpr int CP = BN + 8;
    constexpr int IDX_OFF = (fast_smem_bytes<A_WORDS, B_WORDS, BM, BN, RING>() - (BM + BN) * 4) / 4;

    extern __shared__ __align__(16) uint32_t smem[];
    int* idxA = (int*)(smem + IDX_OFF);
    int* idxB = idxA + BM;
    int* row_list = idxB + BN;          // ring loaders with a row list on the contraction axis

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l32 = lane & 31;
    const int grp = lane >> 5;
    const int wr0 = (wave / WN) * (BM / WM);
    const int wc0 = (wave % WN) * (BN / WN);
    typename LA::Reader ra;
    typename LB::Reader rb;
    if constexpr (M16) { ra.setup16(wr0, lane); rb.setup16(wc0, lane); }
    else { ra.setup(wr0, lane); rb.setup(wc0, lane); }
    // where this lane's accumulator r of result tile (a, b) lies in the workgroup tile
    auto acc_row = [&](int a, int r) {
        return M16 ? wr0 + a * 16 + 4 * (lane >> 4) + r : wr0 + a * 32 + (r >> 2) * 8 + grp * 4 + (r & 3);
    };
    auto acc_col = [&](int b) { return M16 ? wc0 + b * 16 + (lane & 15) : wc0 + b * 32 + l32; };

    // Workgroups go round-robin to the 8 XCDs (each with its own L2): give every
    // XCD a contiguous range of tiles, ordered in groups of 4 tile-rows so that
    // the tiles running together share A rows and B columns.
    const int nb = gridDim.x;                  // a multiple of 8 (the host pads the grid)
    const int per = nb / 8;
    const int lin = (blockIdx.x % 8) * per + blockIdx.x / 8;
    const int total = g.tiles_i * g.tiles_j;
    // phase 1 of a split contraction: slice z of tile t; all tiles of a slice are neighbours in
    // the launch order, so they still sweep the same contraction range together
    const int z = PHASE == 1 ? lin / total : 0;
    const int t = PHASE == 1 ? lin - z * total : lin;
    if (lin >= total * (PHASE == 1 ? g.split : 1)) return;
    constexpr int GI = 4;
    const int grp_sz = GI * g.tiles_j;
    const int gidx = t / grp_sz;
    const int first_i = gidx * GI;
    const int rows_in = min(GI, g.tiles_i - first_i);
    const int within = t - gidx * grp_sz;
    const int ti = first_i + within % rows_in;
    const int tj = within / rows_in;
    const int i0 = g.i_base + ti * BM, j0 = g.j_base + tj * BN;

    if (LA::NEEDS_IDX) {
        const int cnt = min(BM, g.I - i0);
        for (int q = tid; q < cnt; q += NT) idxA[q] = clamp_idx(g.A.map_c[i0 + q], g.A.n_c);
    }
    if (LB::NEEDS_IDX) {
        const int cnt = min(BN, g.J - j0);
        for (int q = tid; q < cnt; q += NT) idxB[q] = clamp_idx(g.B.map_c[j0 + q], g.B.n_c);
    }
    if (LA::NEEDS_IDX || LB::NEEDS_IDX) __syncthreads();

    // The scatter epilogues need the tile's entries of the kept list (one per thread)
    // and the next tile's first entry.  They are requested here and only looked at
    // after the main loop, so their latency never shows.
    static_assert(BM <= NT && BN <= NT, "one kept-list entry per thread");
    // (Unconditional loads: a conditional one would leave a join whose register copies
    // wait for the load right here.  Without a scatter epilogue the address is any
    // readable one, the output's first word, and the value is ignored.)
    const bool scatter_c = g.epilogue == EPI_COL_SCATTER, scatter_r = g.epilogue == EPI_ROW_SCATTER;
    const int k_first = scatter_c ? j0 : i0, k_count = scatter_c ? g.J : g.I, k_tile = scatter_c ? BN : BM;
    const int32_t* k_list = (scatter_c || scatter_r) ? g.keep : (const int32_t*)g.out;
    const int k_last = (scatter_c || scatter_r) ? k_count - 1 : 0;
    const int keep_mine = k_list[min(k_first + tid, k_last)];
    const int keep_next = k_list[min(k_first + k_tile, k_last)];

    ACC acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int r = 0; r < AR; ++r) acc[a][b][r] = 0.f;
    if (g.accumulate) {
        // the accumulators start from the old contents of the output (one rounding
        // at the end); done here, where no other registers are live yet
        const int rows_in_tile = min(BM, g.I - i0), cols_in_tile = min(BN, g.J - j0);
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b)
#pragma unroll
                for (int r = 0; r < AR; ++r) {
                    // coordinates clamped into the tile instead of a guard: the loads need no
                    // branches and go out together; accumulators outside the tile are never stored
                    const int row = min(acc_row(a, r), rows_in_tile - 1);
                    const int col = min(acc_col(b), cols_in_tile - 1);
                    acc[a][b][r] = bf16_bits_to_f32(g.out[(size_t)(i0 + row) * (size_t)g.ldo + j0 + col]);
                }
    }

    // this workgroup's share of the contraction, in 64-deep tiles
    const int KT_all = (g.C + BK - 1) / BK;
    const int kt0 = PHASE == 1 ? z * g.kt_per : 0;
    const int kt1 = PHASE == 1 ? min(kt0 + g.kt_per, KT_all) : KT_all;
    // accumulator sub-tiles (a, b) of this wavefront that hold anything of the output: the
    // slices of a split contraction are only exchanged for those
    auto sub_valid = [&](int a, int b) {
        return wr0 + a * MT < min(BM, g.I - i0) && wc0 + b * MT < min(BN, g.J - j0);
    };
    float4* part = nullptr;
    if constexpr (M16 && PHASE != 0)
        part = (float4*)g.partial + ((size_t)z * (size_t)total + (size_t)t) * (size_t)(TM * TN * NT) + tid;

    LA la;
    LB lb;
    if constexpr (PHASE == 2) {
        // the slices in slice order (a fixed order: results are repeatable bit by bit)
        if constexpr (M16) {
            const size_t zstride = (size_t)total * (size_t)(TM * TN * NT);
            const bool whole_tile = g.I - i0 >= BM && g.J - j0 >= BN;       // uniform over the workgroup
            if (TM * TN <= 16 && whole_tile) {
                // a whole tile: two slices of ALL sub-tiles are requested before any is added (one
                // memory latency per pair of slices; 19 -> 11-16 us per launch on the workload's
                // shapes).  Same order of additions as below.
                for (int z0 = 0; z0 < g.split; z0 += 2) {
                    float4 v[2][TM][TN];
#pragma unroll
                    for (int zz = 0; zz < 2; ++zz)
#pragma unroll
                        for (int a = 0; a < TM; ++a)
#pragma unroll
                            for (int b = 0; b < TN; ++b)
                                v[zz][a][b] = part[(size_t)min(z0 + zz, g.split - 1) * zstride + (a * TN + b) * NT];
#pragma unroll
                    for (int zz = 0; zz < 2; ++zz) {
                        if (z0 + zz >= g.split) break;
#pragma unroll
                        for (int a = 0; a < TM; ++a)
#pragma unroll
                            for (int b = 0; b < TN; ++b) {
                                acc[a][b][0] += v[zz][a][b].x; acc[a][b][1] += v[zz][a][b].y;
                                acc[a][b][2] += v[zz][a][b].z; acc[a][b][3] += v[zz][a][b].w;
                            }
                    }
                }
            } else
            // a tile at the edge (a panel of a few columns, say): all slices of a sub-tile are requested
            // together (one memory latency per sub-tile that holds output, not one per slice) and added
            // in slice order; split <= 8.  (The scheme above measured slower here: 9 -> 12-13 us.)
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b)
                    if (sub_valid(a, b)) {
                        float4 v[8];
#pragma unroll
                        for (int zz = 0; zz < 8; ++zz)
                            v[zz] = part[(size_t)min(zz, g.split - 1) * zstride + (a * TN + b) * NT];
#pragma unroll
                        for (int zz = 0; zz < 8; ++zz)
                            if (zz < g.split) {
                                acc[a][b][0] += v[zz].x; acc[a][b][1] += v[zz].y; acc[a][b][2] += v[zz].z; acc[a][b][3] += v[zz].w;
                            }
                    }
        }
    } else if constexpr (RING) {
        if constexpr (LA::MAPPED || LB::MAPPED) {
            // the row list of the contraction axis, clamped, for the loads of every stage
            const FOp& lop = LA::MAPPED ? g.A : g.B;
            for (int c = tid; c < g.C; c += NT) row_list[c] = clamp_idx(lop.map_s[c], lop.n_s);
            __syncthreads();
        }
        la.init(g.A, i0, g.I, tid, row_list, g.C);
        lb.init(g.B, j0, g.J, tid, row_list, g.C);
        if constexpr (M16) ring_main<LA, LB, TM, TN>(la, lb, ra, rb, g, smem, 2 * kt0, 2 * (kt1 - kt0), acc);
    } else {
        la.init(g.A, i0, g.I, tid, idxA, g.C);
        lb.init(g.B, j0, g.J, tid, idxB, g.C);
        if constexpr (LA::DMA && LB::DMA) {      // (the host only splits products of these loaders)
            if (kt0 > 0) { la.seek(g.A, kt0 * BK, g.C, tid); lb.seek(g.B, kt0 * BK, g.C, tid); }
        }

        // Pipeline over the contraction tiles: while tile k is multiplied out of one LDS
        // stage, tile k+1 travels: direct-to-LDS loaders write it straight into
        // the other stage, register-staged loaders hold it in registers and write
        // it at the end of the iteration.
        auto start_tile = [&](int kt, uint32_t* stage) {
            if constexpr (LA::DMA) la.issue(g.A, stage, kt * BK, g.C, tid); else la.fetch(g.A, kt * BK, g.C, tid);
            if constexpr (LB::DMA) lb.issue(g.B, stage + A_WORDS, kt * BK, g.C, tid); else lb.fetch(g.B, kt * BK, g.C, tid);
        };
        auto finish_tile = [&](uint32_t* stage) {
            if constexpr (LA::DMA) la.settle(g.A);
            if constexpr (LB::DMA) lb.settle(g.B);
            if constexpr (!LA::DMA) la.commit(g.A, stage, tid);
            if constexpr (!LB::DMA) lb.commit(g.B, stage + A_WORDS, tid);
            // direct-to-LDS loads are only tracked by the vector-memory counter: vmcnt(0)
            if constexpr (LA::DMA || LB::DMA) __builtin_amdgcn_s_waitcnt(0x0f70);
        };
        start_tile(kt0, smem);
        finish_tile(smem);
        __syncthreads();

        for (int kt = kt0; kt < kt1; ++kt) {
            const int cur = (kt - kt0) & 1;
            pipeline_step<LA, LB, TM, TN, ACC>(la, lb, ra, rb, g, smem + cur * STAGE_WORDS, smem + (cur ^ 1) * STAGE_WORDS,
                                          (kt + 1) * BK, kt + 1 < kt1, tid, acc);
            __syncthreads();
        }
    }

    if constexpr (PHASE == 1) {
        // this slice's accumulators, as they are; phase 2 adds the slices and stores the output
        if constexpr (M16) {
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b)
                    if (sub_valid(a, b))
                        part[(a * TN + b) * NT] = make_float4(acc[a][b][0], acc[a][b][1], acc[a][b][2], acc[a][b][3]);
        }
        return;
    }

    // ---- epilogue -------------------------------------------------------------
    E* Cs = (E*)smem;
    const int rows_valid = min(BM, g.I - i0);
    const int cols_valid = min(BN, g.J - j0);
    E* out = g.out;
    // accumulators -> C tile in LDS, one column per kept index ("compacted")
    auto stage_compacted = [&] {
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b)
#pragma unroll
                for (int r = 0; r < AR; ++r) Cs[acc_row(a, r) * CP + acc_col(b)] = to_bf16(acc[a][b][r]);
    };

    if (g.epilogue == EPI_COL_SCATTER) {
        // The tile owns the original columns from its first kept column (0 for the
        // first tile) up to the next tile's first kept column (the full width for
        // the last one).
        if (tid < cols_valid) idxB[tid] = clamp_idx(keep_mine, g.out_full);
        __syncthreads();
        const int start = j0 == 0 ? 0 : idxB[0];
        const int end = j0 + BN >= g.J ? g.out_full : clamp_idx(keep_next, g.out_full);

        // Main form: the tile is laid out in LDS the way it lies in memory, one LDS
        // column per ORIGINAL column from `start` (rounded down to a 16-byte chunk) to
        // `end`, half of the tile's rows at a time.  The rows are first filled with the
        // imputed value (+0, or the previous tensor's 16-byte chunks), then every
        // accumulator is written at its original column, then the rows leave with
        // whole 16-byte stores like a plain tile; only the first and last chunk, which
        // the tile shares with its neighbours, are stored element by element.
        constexpr int HR = BM / 2;
        static_assert(HR % 32 == 0, "an MFMA result tile must lie in one half");
        constexpr int MAIN_HALFWORDS = (fast_smem_bytes<A_WORDS, B_WORDS, BM, BN, RING>() - (BM + BN) * 4) / 2;
        const int a0 = start & ~7;
        const int nchunks = (((end + 7) & ~7) - a0) >> 3;
        const int pitch = nchunks * 8 + 8;
        if (g.out_full % 8 == 0 && HR * pitch <= MAIN_HALFWORDS) {
            E* Co = (E*)smem;
            int pos[TN];                       // LDS column of this lane's accumulators, -1 beyond the tile
#pragma unroll
            for (int b = 0; b < TN; ++b) {
                const int col = acc_col(b);
                // (clamped into the row: a list that is not ascending must not leave the tile)
                pos[b] = col < cols_valid ? min(max(idxB[col] - a0, 0), nchunks * 8 - 1) : -1;
            }
            for (int h = 0; h < 2; ++h) {
                const int hr0 = h * HR;
                const int hrows = min(HR, rows_valid - hr0);
                if (hrows <= 0) break;
                for (int u = tid; u < hrows * nchunks; u += NT) {
                    const int r = u / nchunks, c = u - r * nchunks;
                    uint4 v = zero4();
                    if (g.prev) v = *(const uint4*)(g.prev + (size_t)(i0 + hr0 + r) * (size_t)g.ldo + a0 + c * 8);
                    *(uint4*)(Co + r * pitch + c * 8) = v;
                }
                __syncthreads();
#pragma unroll
                for (int a = 0; a < TM; ++a) {
                    if ((wr0 + a * MT) / HR != h) continue;
#pragma unroll
                    for (int b = 0; b < TN; ++b) {
                        if (pos[b] < 0) continue;
#pragma unroll
                        for (int r = 0; r < AR; ++r) Co[(acc_row(a, r) - hr0) * pitch + pos[b]] = to_bf16(acc[a][b][r]);
                    }
                }
                __syncthreads();
                if (g.avg_partial) {
                    // sum of the row's stored (rounded) results; the imputed zeros add nothing
                    float* dst = g.avg_partial + (size_t)(g.avg_slot_base + tj) * (size_t)g.avg_len + i0 + hr0;
                    for (int r = tid; r < hrows; r += NT) {
                        float sum = 0.f;
                        for (int c = start - a0; c < end - a0; ++c) sum += bf16_bits_to_f32(Co[r * pitch + c]);
                        dst[r] = sum;
                    }
                }
                for (int u = tid; u < hrows * nchunks; u += NT) {
                    const int r = u / nchunks, c = u - r * nchunks;
                    const int p = a0 + c * 8;
                    E* o = out + (size_t)(i0 + hr0 + r) * (size_t)g.ldo + p;
                    const E* src = Co + r * pitch + c * 8;
                    if (p >= start && p + 8 <= end) *(uint4*)o = *(const uint4*)src;
                }
                // the first and the last chunk are shared with the neighbouring tiles: their
                // owned elements go out one by one, one work item per (row, element), so
                // that no wavefront serialises on a few lanes
                const int e1_lo = start, e1_hi = (a0 < start || a0 + 8 > end) ? min(end, a0 + 8) : start;
                const int last = a0 + (nchunks - 1) * 8;
                const int e2_lo = max(start, last), e2_hi = (nchunks > 1 && last + 8 > end) ? end : e2_lo;
                const int n1 = e1_hi - e1_lo, ne = n1 + (e2_hi - e2_lo);
                for (int u = tid; u < hrows * ne; u += NT) {
                    const int r = u / ne, e = u - r * ne;
                    const int p = e < n1 ? e1_lo + e : e2_lo + (e - n1);
                    out[(size_t)(i0 + hr0 + r) * (size_t)g.ldo + p] = Co[r * pitch + p - a0];
                }
                __syncthreads();               // the next half reuses the rows
            }
            return;
        }

        // Fallback for tiles that own too many columns for the layout above (sparse kept
        // sets): compacted C tile; work item <-> one aligned pair of original columns
        // over one of RG row groups, consecutive threads on consecutive pairs.
        stage_compacted();
        __syncthreads();
        if (g.avg_partial) {
            // sum of this tile's stored (rounded) results per output row, in column order
            float* dst = g.avg_partial + (size_t)(g.avg_slot_base + tj) * (size_t)g.avg_len + i0;
            for (int row = tid; row < rows_valid; row += NT) {
                float sum = 0.f;
                for (int c = 0; c < cols_valid; ++c) sum += bf16_bits_to_f32(Cs[row * CP + c]);
                dst[row] = sum;
            }
        }
        constexpr int RG = 8;
        constexpr int ROWS_PER = (BM + RG - 1) / RG;
        const int first = start & ~1;
        const int npairs = (end - first + 1) >> 1;
        for (int item = tid; item < npairs * RG; item += NT) {
            const int rg = item / npairs;
            const int pbase = first + 2 * (item - rg * npairs);
            const int row_lo = rg * ROWS_PER, row_hi = min(rows_valid, row_lo + ROWS_PER);
            const int p0 = pbase, p1 = pbase + 1;
            const bool own0 = p0 >= start, own1 = p1 < end;
            int r0 = lower_bound_lds(idxB, cols_valid, p0);
            const bool k0 = own0 && r0 < cols_valid && idxB[r0] == p0;
            int r1 = r0 + ((r0 < cols_valid && idxB[r0] == p0) ? 1 : 0);
            const bool k1 = own1 && r1 < cols_valid && idxB[r1] == p1;
            r0 = k0 ? r0 : 0;
            r1 = k1 ? r1 : 0;
            E* o = out + (size_t)i0 * (size_t)g.ldo + p0;
            if (!g.prev) {
                // dropped positions receive +0
                if (own0 && own1) {
                    // 8 rows at a time: all LDS reads go out before the first store,
                    // so the loop pays one LDS round trip per 8 rows
                    constexpr int UB = 8;
                    for (int row = row_lo; row < row_hi; row += UB) {
                        uint32_t v[UB];
#pragma unroll
                        for (int u = 0; u < UB; ++u) {
                            const int rr_ = min(row + u, row_hi - 1);
                            const uint32_t v0 = k0 ? Cs[rr_ * CP + r0] : 0u;
                            const uint32_t v1 = k1 ? Cs[rr_ * CP + r1] : 0u;
                            v[u] = v0 | (v1 << 16);
                        }
#pragma unroll
                        for (int u = 0; u < UB; ++u)
                            if (row + u < row_hi) *(uint32_t*)(o + (size_t)(row + u) * (size_t)g.ldo) = v[u];
                    }
                } else if (own0) {
                    for (int row = row_lo; row < row_hi; ++row)
                        o[(size_t)row * (size_t)g.ldo] = k0 ? Cs[row * CP + r0] : E(0);
                } else if (own1) {
                    for (int row = row_lo; row < row_hi; ++row)
                        o[(size_t)row * (size_t)g.ldo + 1] = k1 ? Cs[row * CP + r1] : E(0);
                }
                continue;
            }
            // Same: dropped positions copy the previous tensor's value.  The previous tensor
            // may be the output itself, but a position is only ever read and written by this
            // thread, so the loads of a batch of rows may all go out before its stores
            // (one load latency per batch instead of one per row).
            const E* pv = g.prev + (size_t)i0 * (size_t)g.ldo + p0;
            constexpr int RB = 16;
            if (own0 && own1) {
                const bool need_prev = !(k0 && k1);
                for (int row = row_lo; row < row_hi; row += RB) {
                    uint32_t old[RB];
#pragma unroll
                    for (int u = 0; u < RB; ++u)
                        old[u] = (need_prev && row + u < row_hi)
                                     ? *(const uint32_t*)(pv + (size_t)(row + u) * (size_t)g.ldo) : 0u;
#pragma unroll
                    for (int u = 0; u < RB; ++u) {
                        if (row + u >= row_hi) break;
                        const uint32_t v0 = k0 ? Cs[(row + u) * CP + r0] : (old[u] & 0xffffu);
                        const uint32_t v1 = k1 ? Cs[(row + u) * CP + r1] : (old[u] >> 16);
                        *(uint32_t*)(o + (size_t)(row + u) * (size_t)g.ldo) = v0 | (v1 << 16);
                    }
                }
            } else if (own0 || own1) {
                const int side = own0 ? 0 : 1;
                const bool kept = own0 ? k0 : k1;
                const int rr = own0 ? r0 : r1;
                for (int row = row_lo; row < row_hi; row += RB) {
                    E old[RB];
#pragma unroll
                    for (int u = 0; u < RB; ++u)
                        old[u] = (!kept && row + u < row_hi) ? pv[(size_t)(row + u) * (size_t)g.ldo + side] : E(0);
#pragma unroll
                    for (int u = 0; u < RB; ++u) {
                        if (row + u >= row_hi) break;
                        o[(size_t)(row + u) * (size_t)g.ldo + side] = kept ? Cs[(row + u) * CP + rr] : old[u];
                    }
                }
            }
        }
        return;
    }

    stage_compacted();
    const bool scatter_rows = g.epilogue == EPI_ROW_SCATTER;
    if (scatter_rows && tid < rows_valid) idxA[tid] = clamp_idx(keep_mine, g.out_full);
    __syncthreads();
    if (scatter_rows && g.avg_partial) {
        // sum of this tile's stored (rounded) results per output column, in row order
        float* dst = g.avg_partial + (size_t)(g.avg_slot_base + ti) * (size_t)g.avg_len + j0;
        for (int col = tid; col < cols_valid; col += NT) {
            float sum = 0.f;
            for (int r = 0; r < rows_valid; ++r) sum += bf16_bits_to_f32(Cs[r * CP + col]);
            dst[col] = sum;
        }
    }
    constexpr int CPR = BN / 8;
    for (int q = tid; q < BM * CPR; q += NT) {
        const int row = q / CPR;
        const int j = (q % CPR) * 8;
        if (row >= rows_valid || j >= cols_valid) continue;      // J is a multiple of 8 on this path
        const int orow = scatter_rows ? idxA[row] : i0 + row;
        *(uint4*)(out + (size_t)orow * (size_t)g.ldo + j0 + j) = *(const uint4*)(Cs + row * CP + j);
    }
    if (scatter_rows) {
        const int start = i0 == 0 ? 0 : idxA[0];
        const int end = i0 + BM >= g.I ? g.out_full : clamp_idx(keep_next, g.out_full);
        // Which of the rows [start, end) are dropped: every lane looks one row up (64
        // searches side by side instead of one after the other), then the wavefront
        // walks the set bits of the ballot and writes each dropped row together.
        for (int base = start + wave * 64; base < end; base += NT) {
            const int mine = base + lane;
            bool dropped = false;
            if (mine < end) {
                const int ii = lower_bound_lds(idxA, rows_valid, mine);
                dropped = !(ii < rows_valid && idxA[ii] == mine);
            }
            unsigned long long todo = __ballot(dropped);
            while (todo) {
                const int p = base + (__ffsll((long long)todo) - 1);
                todo &= todo - 1;
                E* o = out + (size_t)p * (size_t)g.ldo + j0;
                if (!g.prev) {
                    for (int j = lane * 8; j < cols_valid; j += 64 * 8) *(uint4*)(o + j) = zero4();
                } else {
                    const E* pv = g.prev + (size_t)p * (size_t)g.ldo + j0;
                    for (int j = lane * 8; j < cols_valid; j += 64 * 8) *(uint4*)(o + j) = *(const uint4*)(pv + j);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
// ZR_NO_SPLIT in the environment (read once) switches the split contraction off: an A/B switch.
inline bool split_enabled()
{
    static const bool on = getenv("ZR_NO_SPLIT") == nullptr;
    return on;
}

template <template <int, int> class LA, template <int, int> class LB, int BM, int BN, int WM, int WN>
int launch_inst(const FArgs& a, int i_base, int i_end, int j_base, int j_end, hipStream_t stream, int slot_base)
{
    typedef LA<BM, 64 * WM * WN> A;
    typedef LB<BN, 64 * WM * WN> B;
    constexpr bool ring = A::RING;
    constexpr int list_bytes = [] { if constexpr (ring) return (A::MAPPED || B::MAPPED) ? ring_list_max<BM, BN>() * 4 : 0; else return 0; }();
    constexpr int smem = fast_smem_bytes<A::WORDS, B::WORDS, BM, BN, ring>() + list_bytes;
    static_assert(smem <= 160 * 1024, "LDS of a workgroup");
    auto fn = fast_kernel<LA, LB, BM, BN, WM, WN>;
    static AttrFlags attr_set;      // per instantiation and device
    if (!ensure_max_dynamic_lds((const void*)fn, smem, &attr_set)) return ZR_ERR_HIP;
    if (debug_names_wanted())
        snprintf(g_debug.last_kernel, sizeof(g_debug.last_kernel), "fast_kernel<%s, %s, %d, %d, %d, %d>",
                 A::NAME, B::NAME, BM, BN, WM, WN);
    FArgs k = a;
    k.i_base = i_base; k.i_end = i_end; k.j_base = j_base; k.j_end = j_end;
    k.avg_slot_base = slot_base;
    k.tiles_i = (i_end - i_base + BM - 1) / BM;
    k.tiles_j = (j_end - j_base + BN - 1) / BN;
    const int64_t tiles = (int64_t)k.tiles_i * k.tiles_j;
    if (tiles > 0x7ffffff0) return ZR_ERR_LIMIT;
    k.phase = 0; k.split = 1; k.kt_per = 0;
    // Split contraction: when this launch has too few tiles for the chip and a long contraction,
    // s slices per tile (s * tiles workgroups), then one more launch of the same kernel that adds
    // the slices and runs the epilogue.  Needs scratch for the slices (the caller's workspace).
    // (Tried on the big ring tiles of the dW products at high pruning ratios as well, 128 tiles
    // of 192 x 256 in two slices each: the slices are 50 MB of fp32 that leave the chip at the
    // end of the first launch and come back in the second, ~35 us per product, which is all
    // that the better fill of the chip gains.  Not instantiated.)
    constexpr bool can_split = A::DMA && B::DMA && !ring && BM == 128 && BN == 128;
    if constexpr (can_split) {
        const int KT = (a.C + BK - 1) / BK;
        const int64_t slots = (BM * BN > 128 * 128) ? 256 : 512;          // workgroups the chip holds at once
        int sp = (int)std::min<int64_t>(slots / tiles, 8);
        sp = std::min(sp, KT / 8);                                         // at least 8 contraction tiles (512 deep) per slice
        const size_t per_slice = (size_t)tiles * (size_t)BM * (size_t)BN * 4;
        if (a.partial && per_slice > 0) sp = (int)std::min<size_t>((size_t)std::max(sp, 0), a.partial_bytes / per_slice);
        else sp = 1;
        if (sp >= 2 && !a.accumulate && split_enabled()) {
            k.split = sp; k.kt_per = (KT + sp - 1) / sp;
            k.split = (KT + k.kt_per - 1) / k.kt_per;                      // no empty slice
            auto fn1 = fast_kernel<LA, LB, BM, BN, WM, WN, 1>;
            auto fn2 = fast_kernel<LA, LB, BM, BN, WM, WN, 2>;
            static AttrFlags attr1, attr2;
            if (!ensure_max_dynamic_lds((const void*)fn1, smem, &attr1) || !ensure_max_dynamic_lds((const void*)fn2, smem, &attr2))
                return ZR_ERR_HIP;
            k.phase = 1;
            const int64_t g1 = (tiles * k.split + 7) / 8 * 8;
            hipLaunchKernelGGL(fn1, dim3((unsigned)g1), dim3(64 * WM * WN), smem, stream, k);
            if (hipGetLastError() != hipSuccess) return ZR_ERR_HIP;
            k.phase = 2;
            hipLaunchKernelGGL(fn2, dim3((unsigned)((tiles + 7) / 8 * 8)), dim3(64 * WM * WN), smem, stream, k);
            if (debug_names_wanted()) {
                char nm[128];
                snprintf(nm, sizeof(nm), "%.90s split %d", g_debug.last_kernel, k.split);
                snprintf(g_debug.last_kernel, sizeof(g_debug.last_kernel), "%s", nm);
            }
            return hip_status(hipGetLastError());
        }
    }
    const int64_t grid = (tiles + 7) / 8 * 8;
    hipLaunchKernelGGL(fn, dim3((unsigned)grid), dim3(64 * WM * WN), smem, stream, k);
    return hip_status(hipGetLastError());
}

// ZR_NO_RING in the environment (read once) keeps every product on the 64-deep two-stage loop:
// an A/B switch for measurements.
inline bool ring_enabled()
{
    static const bool on = getenv("ZR_NO_RING") == nullptr;
    return on;
}

template <template <int, int> class LA, template <int, int> class LB, int BM, int BN, int WM, int WN>
int launch_tile(const FArgs& a, int i_base, int i_end, int j_base, int j_end, hipStream_t stream, int slot_base = 0)
{
    if (i_end <= i_base || j_end <= j_base) return ZR_OK;
    if constexpr (RingOf<LA>::has && RingOf<LB>::has) {
        constexpr int NT = 64 * WM * WN;
        typedef typename RingOf<LA>::template type<BM, NT> RA;
        typedef typename RingOf<LB>::template type<BN, NT> RB;
        constexpr int TM = BM / (16 * WM), TN = BN / (16 * WN);
        constexpr int ring_a = TM % 4 == 0 ? 4 : 3;
        // the ring schedule needs whole load instructions per wavefront and enough MFMA slots
        // (and tiles above 128 x 128: the small tiles, four wavefronts and two workgroups to a compute
        // unit, measured 10-25 % slower with a barrier every 32 instead of every 64)
        constexpr bool fits = RA::FITS && RB::FITS && TM % ring_a == 0 && TM >= 4 && TN >= 4 && RA::NI + RB::NI <= TM &&
                              (TN <= TM - 1 || 2 * (TM - 1) >= TN) && BM * BN > 128 * 128;
        if constexpr (fits) {
            const bool list_ok = !(RA::MAPPED || RB::MAPPED) || a.C <= ring_list_max<BM, BN>();
            if (ring_enabled() && list_ok) {
                // (named directly, so that a profiler prints the loaders' own names)
                constexpr bool ap = std::is_same<RA, RingP<BM, NT>>::value, aq = std::is_same<RA, RingQ<BM, NT>>::value;
                constexpr bool bp = std::is_same<RB, RingP<BN, NT>>::value, bq = std::is_same<RB, RingQ<BN, NT>>::value;
                constexpr bool bm = std::is_same<RB, RingQM<BN, NT>>::value;
                static_assert((ap && (bp || bq || bm)) || (aq && bq), "loader pair without a ring instantiation");
                if constexpr (ap && bp) return launch_inst<RingP, RingP, BM, BN, WM, WN>(a, i_base, i_end, j_base, j_end, stream, slot_base);
                else if constexpr (ap && bq) return launch_inst<RingP, RingQ, BM, BN, WM, WN>(a, i_base, i_end, j_base, j_end, stream, slot_base);
                else if constexpr (ap && bm) return launch_inst<RingP, RingQM, BM, BN, WM, WN>(a, i_base, i_end, j_base, j_end, stream, slot_base);
                else return launch_inst<RingQ, RingQ, BM, BN, WM, WN>(a, i_base, i_end, j_base, j_end, stream, slot_base);
            }
        }
    }
    return launch_inst<LA, LB, BM, BN, WM, WN>(a, i_base, i_end, j_base, j_end, stream, slot_base);
}

// Tile schedule.  The chip has 256 CUs; a 256 x 256 tile occupies one CU (one
// "round" = 256 such tiles), two 128 x 128 tiles share a CU.  A grid whose tile
// count is just above a multiple of 256 would leave most CUs idle in its last
// round, so D is cut into a panel of big tiles that fills whole rounds and a
// remainder panel of small tiles (a second launch), whichever cut of rows or
// columns is estimated cheapest.  Costs are in units of one big-tile round;
// the constants come from measurements on the workload shapes.
struct Sched {
    int big_i_end, big_j_end;   // big tiles cover [0, big_i_end) x [0, big_j_end); 0 = no big panel
    bool cut_rows;              // the remainder panel is rows [big_i_end, I) (else columns [big_j_end, J))
    double cost;                // estimate, in big-tile rounds
};

// One grid of 256 x 192 (or 192 x 256) tiles: three quarters of the MFMA work of a
// big tile but 0.84 of its LDS traffic, which is what bounds the loop.  Only the
// direct-to-LDS loaders have this shape.
#ifndef ZR_COST_192
#define ZR_COST_192 0.85
#endif
inline int64_t tiles_of(int I, int J, int bm, int bn) { return (int64_t)((I + bm - 1) / bm) * ((J + bn - 1) / bn); }
inline double cost_192(int64_t tiles) { return ZR_COST_192 * (double)((tiles + 255) / 256); }

#ifndef ZR_COST_SMALL1
#define ZR_COST_SMALL1 0.46
#endif
#ifndef ZR_COST_SMALL2
#define ZR_COST_SMALL2 0.77
#endif
#ifndef ZR_COST_SPLIT
#define ZR_COST_SPLIT 0.30
#endif
inline double small_cost(int64_t ts)
{
    if (ts <= 0) return 0.0;
    if (ts <= 128) return ZR_COST_SPLIT;                        // few tiles: the contraction is split (with scratch)
    if (ts <= 256) return ZR_COST_SMALL1;                       // one small tile per CU
    return ZR_COST_SMALL2 * (double)((ts + 511) / 512);         // two per CU
}

inline Sched plan_tiles(int I, int J)
{
    const int ti = (I + 255) / 256, tj = (J + 255) / 256;
    const int64_t T = (int64_t)ti * tj;
    auto smalls = [](int rows, int cols) { return (int64_t)((rows + 127) / 128) * ((cols + 127) / 128); };
    Sched best{I, J, true, 0.0};
    double best_cost = (double)((T + 255) / 256);                  // all big
    {
        const double c = small_cost(smalls(I, J));                 // all small
        if (c < best_cost) { best_cost = c; best = Sched{0, 0, true, 0.0}; }
    }
    for (int q = 1; q * 256 < T; ++q) {                            // q full rounds of big tiles
        const int rb = (int)((int64_t)q * 256 / tj);               // big tile-rows
        if (rb >= 1 && rb < ti) {
            const double c = (double)(((int64_t)rb * tj + 255) / 256) + small_cost(smalls(I - rb * 256, J));
            if (c < best_cost) { best_cost = c; best = Sched{rb * 256, J, true, 0.0}; }
        }
        const int cb = (int)((int64_t)q * 256 / ti);               // big tile-columns
        if (cb >= 1 && cb < tj) {
            const double c = (double)(((int64_t)cb * ti + 255) / 256) + small_cost(smalls(I, J - cb * 256));
            if (c < best_cost) { best_cost = c; best = Sched{I, cb * 256, false, 0.0}; }
        }
    }
    best.cost = best_cost;
    return best;
}

// ZR_FORCE_TILES in the environment (read once): "256", "192x256" or "256x192" sends every product
// of this path to one grid of that tile shape, whatever the schedule would choose: a test switch
// (small and ragged shapes then run through the big-tile kernels).  0 = not set.
inline int forced_tiles()
{
    static const int f = [] {
        const char* e = getenv("ZR_FORCE_TILES");
        if (!e) return 0;
        if (!strcmp(e, "256")) return 1;
        if (!strcmp(e, "192x256")) return 2;
        if (!strcmp(e, "256x192")) return 3;
        return 0;
    }();
    return f;
}

template <template <int, int> class LA, template <int, int> class LB>
int launch_shape(const FArgs& a, hipStream_t stream)
{
    if (const int f = forced_tiles()) {
        if constexpr (LA<256, 512>::DMA && LB<256, 512>::DMA) {
            if (f == 2) return launch_tile<LA, LB, 192, 256, 2, 4>(a, 0, a.I, 0, a.J, stream);
            if (f == 3) return launch_tile<LA, LB, 256, 192, 4, 2>(a, 0, a.I, 0, a.J, stream);
        }
        return launch_tile<LA, LB, 256, 256, ZR_BIG_WM, ZR_BIG_WN>(a, 0, a.I, 0, a.J, stream);
    }
    const Sched sc = plan_tiles(a.I, a.J);
    if constexpr (LA<256, 512>::DMA && LB<256, 512>::DMA) {
        const int64_t tj = tiles_of(a.I, a.J, 256, 192), ti = tiles_of(a.I, a.J, 192, 256);
        const double cj = cost_192(tj), ci = cost_192(ti);
        if (std::min(cj, ci) < sc.cost - 1e-9) {
            // equal rounds: the grid with fewer tiles has less padding
            if (cj < ci || (cj == ci && tj <= ti)) return launch_tile<LA, LB, 256, 192, 4, 2>(a, 0, a.I, 0, a.J, stream);
            return launch_tile<LA, LB, 192, 256, 2, 4>(a, 0, a.I, 0, a.J, stream);
        }
    }
    if (sc.big_i_end == 0)                     // everything on small tiles
        return launch_tile<LA, LB, 128, 128, 2, 2>(a, 0, a.I, 0, a.J, stream);
    int st = launch_tile<LA, LB, 256, 256, ZR_BIG_WM, ZR_BIG_WN>(a, 0, sc.big_i_end, 0, sc.big_j_end, stream);
    if (st != ZR_OK || (sc.big_i_end >= a.I && sc.big_j_end >= a.J)) return st;
    char big[128];
    if (debug_names_wanted()) snprintf(big, sizeof(big), "%s", g_debug.last_kernel);
    // Average sums: the remainder panel's tiles continue the slot numbering of the big
    // panel along the summed axis when the cut runs across that axis; panels that
    // cover different output rows (columns) never meet in a slot
    const bool sums_over_j = a.epilogue == EPI_COL_SCATTER;
    if (sc.cut_rows) st = launch_tile<LA, LB, 128, 128, 2, 2>(a, sc.big_i_end, a.I, 0, a.J, stream,
                                                              sums_over_j ? 0 : sc.big_i_end / 256);
    else st = launch_tile<LA, LB, 128, 128, 2, 2>(a, 0, a.I, sc.big_j_end, a.J, stream,
                                                  sums_over_j ? sc.big_j_end / 256 : 0);
    if (debug_names_wanted())
        snprintf(g_debug.last_kernel, sizeof(g_debug.last_kernel), "%.60s + 128x128 remainder panel", big);
    return st;
}

}  // namespace

// Returns -1 when the problem is not eligible for this path (the caller then
// uses the general kernel), else a zr_status.
int launch_gemm_fast(const GemmDesc& d, hipStream_t stream)
{
    if (d.dtype != ZR_BF16) return -1;
    auto aligned = [](const void* p, int64_t ld) { return ((uintptr_t)p % 16 == 0) && (ld % 8 == 0); };
    if (!aligned(d.A.base, d.A.ld) || !aligned(d.B.base, d.B.ld) || !aligned(d.out, d.ldo)) return -1;
    // every memory row that is walked in 16-byte chunks must be a multiple of 8 long
    auto chunked_ok = [](const Operand& o) {
        if (o.map_contig) {
            if (o.map_strided) return false;
            return o.c_contig ? o.n_contig % 2 == 0 : o.n_contig % 8 == 0;   // PG reads aligned dwords, QG chunks
        }
        return o.n_contig % 8 == 0;
    };
    if (!chunked_ok(d.A) || !chunked_ok(d.B)) return -1;
    if (d.epilogue != EPI_COL_SCATTER && d.J % 8 != 0) return -1;
    if (d.I < 1 || d.J < 1 || d.C < 1) return -1;
    if (d.prev && (uintptr_t)d.prev % 16 != 0) return -1;
    if (d.accumulate && d.epilogue != EPI_PLAIN) return -1;

    FArgs a;
    a.A = FOp{(const E*)d.A.base, d.A.ld, d.A.map_strided, d.A.map_contig, d.A.n_strided, d.A.n_contig};
    a.B = FOp{(const E*)d.B.base, d.B.ld, d.B.map_strided, d.B.map_contig, d.B.n_strided, d.B.n_contig};
    a.I = d.I; a.J = d.J; a.C = d.C;
    a.out = (E*)d.out; a.ldo = d.ldo; a.epilogue = d.epilogue; a.keep = d.keep_idx; a.out_full = d.out_full;
    a.prev = (const E*)d.prev; a.accumulate = d.accumulate ? 1 : 0;
    a.avg_partial = d.epilogue == EPI_PLAIN ? nullptr : d.avg_partial; a.avg_len = d.avg_len; a.avg_slot_base = 0;
    a.tiles_i = a.tiles_j = 0;
    a.i_base = a.j_base = a.i_end = a.j_end = 0;
    a.partial = (float*)d.split_scratch; a.partial_bytes = d.split_scratch ? d.split_scratch_bytes : 0;
    a.split = 1; a.phase = 0; a.kt_per = 0;
    const bool ag = d.A.map_contig != nullptr, bg = d.B.map_contig != nullptr;
    // Direct-to-LDS loaders cannot zero the contraction tail of the last tile
    // themselves: either the tiles are full, or one operand supplies the zeros
    // (a register-staged loader, or a zero-padded extracted activation).
    const bool full_tiles = d.C % BK == 0;
    const bool a_zero = ag || (d.A.c_contig && d.A.zero_padded);
    const bool b_zero = bg || (d.B.c_contig && d.B.zero_padded);
    const bool dma_ok = full_tiles || a_zero || b_zero;
    if (d.A.c_contig && !d.B.c_contig) {            // forward: X rows, W columns
        const bool bm = d.B.map_strided != nullptr;        // W[S[c], :]: the row list is on the contraction axis
        if (!ag && !bg) {
            if (!dma_ok) return launch_shape<LdPV, LdQV>(a, stream);
            return bm ? launch_shape<DmaP, DmaQM>(a, stream) : launch_shape<DmaP, DmaQ>(a, stream);
        }
        if (ag && !bg) return bm ? launch_shape<LdPG, DmaQM>(a, stream) : launch_shape<LdPG, DmaQ>(a, stream);
        if (!ag && bg) return launch_shape<DmaP, LdQG>(a, stream);
        return -1;
    }
    if (d.A.c_contig && d.B.c_contig) {             // dX
        if (!ag && !bg) return dma_ok ? launch_shape<DmaP, DmaP>(a, stream) : launch_shape<LdPV, LdPV>(a, stream);
        if (ag && bg) return launch_shape<LdPG, LdPG>(a, stream);
        if (!ag && bg) return launch_shape<DmaP, LdPG>(a, stream);
        return -1;
    }
    if (!d.A.c_contig && !d.B.c_contig) {           // dW: the contraction runs over the tokens, never through a list
        if (d.A.map_strided || d.B.map_strided) return -1;
        if (!ag && !bg) return full_tiles ? launch_shape<DmaQ, DmaQ>(a, stream) : launch_shape<LdQV, LdQV>(a, stream);
        if (ag && !bg) return launch_shape<LdQG, DmaQ>(a, stream);
        if (!ag && bg) return launch_shape<DmaQ, LdQG>(a, stream);
        return -1;
    }
    return -1;
}

}  // namespace zr

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
//   rows of a tensor (W[S,:])            -> the row list only changes the row
//        pointer of ordinary 16-byte loads (loaders PV / QV).
//   contiguous axis, non-contraction     -> (W[:,S] in forward, X[:,S] and
//        dY[:,S] in dW) the full-width span of the tile's kept columns is
//        fetched with 16-byte loads, two memory rows are interleaved into
//        (c, c+1) words in registers, and only the kept columns' words are
//        written to LDS, at their compacted positions (loader QG).
//   contiguous axis, contraction         -> (X[:,S] in forward DROP_K, dY[:,S]
//        and W[:,S] in dX DROP_N) each LDS word (two consecutive kept indices
//        of one row) is assembled from two aligned dword loads with one byte
//        permute (loader PG).
// The epilogue composes full-width output rows in LDS order: kept columns get
// their result, dropped columns of the tile's span get +0, stored as dwords.
#include "zr_common.h"

namespace zr {

namespace {

constexpr int BK = 64;           // contraction depth of one LDS tile (bf16 elements)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint16_t E;

// LDS tile layout, the same for every operand kind: 8 blocks (one per group of
// 8 contraction indices); inside a block every tile row owns one 16-byte slot
// holding its 8 bf16 of that group, so an MFMA k-vector is one ds_read_b128.
// The LDS serves 16-byte accesses 8 lanes at a time over 32 banks (128 bytes):
// 8 consecutive lanes must hit 8 different slots modulo 8.  Rows are placed at
// slot(i) = i + (i >> 3), which gives that both for 8 consecutive rows (fragment
// reads, row-wise writes) and for rows 8 apart (writes of the loaders whose
// lanes hold 8 consecutive columns each); blocks are 1 slot out of phase so
// that lanes writing the same row of different blocks do not collide either.
template <int R> struct Tile {
    static constexpr int BW = (R + R / 8 + 1) * 4;    // words per block
    static constexpr int WORDS = 8 * BW;
    static __device__ __forceinline__ int slot(int i) { return i + (i >> 3); }
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
    int tiles_i, tiles_j;
};

// fp32 -> bf16, round to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ E to_bf16(float f)
{
    union { __bf16 h; E u; } x;
    x.h = (__bf16)f;
    return x.u;
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
    typedef Tile<R> T;
    static constexpr int N = R * 8 / NT;
    static constexpr bool NEEDS_IDX = false;
    const E* ptr[N];
    uint4 v[N];
    bool ok_;               // the fetched chunk lies inside the contraction range

    __device__ __forceinline__ void init(const FOp& op, int r0, int rlim, int tid, int*, int)
    {
#pragma unroll
        for (int it = 0; it < N; ++it) {
            const int q = tid + NT * it;
            const int i = min(r0 + (q >> 3), rlim - 1);
            const int srow = op.map_s ? clamp_idx(op.map_s[i], op.n_s) : i;
            ptr[it] = op.base + (size_t)srow * (size_t)op.ld + (q & 7) * 8;
        }
    }
    __device__ __forceinline__ void fetch(const FOp&, int c0, int C, int tid)
    {
        const int c = c0 + (tid & 7) * 8;            // C is a multiple of 8 on this path
        ok_ = c < C;
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
    typedef Tile<R> T;
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
    typedef Tile<R> T;
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
#pragma unroll
        for (int it = 0; it < N; ++it) {
            const int c = c0 + 4 * ((tid + NT * it) / UPR);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int cu = min(c + u, C - 1);
                rr[it][u] = op.map_s ? clamp_idx(op.map_s[cu], op.n_s) : cu;
            }
        }
    }
    __device__ __forceinline__ void init(const FOp& op, int r0, int rlim, int tid, int*, int C)
    {
#pragma unroll
        for (int it = 0; it < N; ++it) {
            const int j = min(r0 + ((tid + NT * it) % UPR) * 8, rlim - 8);   // extent is a multiple of 8 here
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
            uint32_t* dst = lds + (kq >> 1) * T::BW + (kq & 1) * 2 + jc * 36;  // slot(8 jc + m) = 9 jc + m
#pragma unroll
            for (int m = 0; m < 8; ++m) *(uint2*)(dst + m * 4) = w[m];
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
    typedef Tile<R> T;
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
__device__ __forceinline__ bf16x8 read_frag(const uint32_t* p)
{
    union { uint4 u; bf16x8 b; } x;
    x.u = *(const uint4*)p;
    return x.b;
}

template <int BM, int BN>
constexpr int fast_smem_bytes()
{
    constexpr int stage_bytes = 2 * (Tile<BM>::WORDS + Tile<BN>::WORDS) * 4;
    constexpr int c_bytes = BM * (BN + 8) * 2;
    return (stage_bytes > c_bytes ? stage_bytes : c_bytes) + (BM + BN) * 4;
}

template <template <int, int> class LA_, template <int, int> class LB_, int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(64 * WM * WN) void fast_kernel(const FArgs g)
{
    constexpr int NT = 64 * WM * WN;
    constexpr int TM = BM / (32 * WM), TN = BN / (32 * WN);
    constexpr int A_WORDS = Tile<BM>::WORDS;
    constexpr int B_WORDS = Tile<BN>::WORDS;
    constexpr int STAGE_WORDS = A_WORDS + B_WORDS;
    constexpr int CP = BN + 8;
    constexpr int IDX_OFF = (fast_smem_bytes<BM, BN>() - (BM + BN) * 4) / 4;
    typedef LA_<BM, NT> LA;
    typedef LB_<BN, NT> LB;

    extern __shared__ __align__(16) uint32_t smem[];
    int* idxA = (int*)(smem + IDX_OFF);
    int* idxB = idxA + BM;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l32 = lane & 31;
    const int grp = lane >> 5;
    const int wr0 = (wave / WN) * (BM / WM);
    const int wc0 = (wave % WN) * (BN / WN);
    // word offset of this lane's first fragment row inside a block; the row 32
    // further down sits 36 slots (144 words) further
    const int arow = Tile<BM>::slot(wr0 + l32) * 4;
    const int brow = Tile<BN>::slot(wc0 + l32) * 4;

    // Workgroups go round-robin to the 8 XCDs (each with its own L2): give every
    // XCD a contiguous range of tiles, ordered in groups of 4 tile-rows so that
    // the tiles running together share A rows and B columns.
    const int nb = gridDim.x;                  // a multiple of 8 (the host pads the grid)
    const int per = nb / 8;
    const int t = (blockIdx.x % 8) * per + blockIdx.x / 8;
    const int total = g.tiles_i * g.tiles_j;
    if (t >= total) return;
    constexpr int GI = 4;
    const int grp_sz = GI * g.tiles_j;
    const int gidx = t / grp_sz;
    const int first_i = gidx * GI;
    const int rows_in = min(GI, g.tiles_i - first_i);
    const int within = t - gidx * grp_sz;
    const int ti = first_i + within % rows_in;
    const int tj = within / rows_in;
    const int i0 = ti * BM, j0 = tj * BN;

    if (LA::NEEDS_IDX) {
        const int cnt = min(BM, g.I - i0);
        for (int q = tid; q < cnt; q += NT) idxA[q] = clamp_idx(g.A.map_c[i0 + q], g.A.n_c);
    }
    if (LB::NEEDS_IDX) {
        const int cnt = min(BN, g.J - j0);
        for (int q = tid; q < cnt; q += NT) idxB[q] = clamp_idx(g.B.map_c[j0 + q], g.B.n_c);
    }
    if (LA::NEEDS_IDX || LB::NEEDS_IDX) __syncthreads();

    f32x16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    LA la;
    LB lb;
    la.init(g.A, i0, g.I, tid, idxA, g.C);
    lb.init(g.B, j0, g.J, tid, idxB, g.C);

    // Software pipeline over the contraction tiles: tile k is multiplied out of
    // LDS stage k&1 while tile k+1 (fetched into registers one iteration
    // earlier) is written to the other stage and the global loads of tile k+2
    // are issued, both in the middle of the MFMA sequence.
    const int KT = (g.C + BK - 1) / BK;
    la.fetch(g.A, 0, g.C, tid);
    lb.fetch(g.B, 0, g.C, tid);
    la.commit(g.A, smem, tid);
    lb.commit(g.B, smem + A_WORDS, tid);
    if (KT > 1) {
        la.fetch(g.A, BK, g.C, tid);
        lb.fetch(g.B, BK, g.C, tid);
    }
    __syncthreads();

    auto mma_step = [&](const uint32_t* as, const uint32_t* bs, int step) {
        // lanes 0-31 take contraction indices 16*step .. +7, lanes 32-63 the next 8
        const uint32_t* ab = as + (2 * step + grp) * Tile<BM>::BW;
        const uint32_t* bb = bs + (2 * step + grp) * Tile<BN>::BW;
        bf16x8 af[TM], bf[TN];
#pragma unroll
        for (int a = 0; a < TM; ++a) af[a] = read_frag(ab + a * 144);
#pragma unroll
        for (int b = 0; b < TN; ++b) bf[b] = read_frag(bb + b * 144);
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bf[b], acc[a][b], 0, 0, 0);
    };

    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        const uint32_t* as = smem + cur * STAGE_WORDS + arow;
        const uint32_t* bs = smem + cur * STAGE_WORDS + A_WORDS + brow;
        mma_step(as, bs, 0);
        mma_step(as, bs, 1);
        if (kt + 1 < KT) {
            la.commit(g.A, smem + (cur ^ 1) * STAGE_WORDS, tid);
            lb.commit(g.B, smem + (cur ^ 1) * STAGE_WORDS + A_WORDS, tid);
        }
        if (kt + 2 < KT) {
            la.fetch(g.A, (kt + 2) * BK, g.C, tid);
            lb.fetch(g.B, (kt + 2) * BK, g.C, tid);
        }
        mma_step(as, bs, 2);
        mma_step(as, bs, 3);
        __syncthreads();
    }

    // ---- epilogue -------------------------------------------------------------
    E* Cs = (E*)smem;
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = wr0 + a * 32 + (r >> 2) * 8 + grp * 4 + (r & 3);
                Cs[row * CP + wc0 + b * 32 + l32] = to_bf16(acc[a][b][r]);
            }
    const int rows_valid = min(BM, g.I - i0);
    const int cols_valid = min(BN, g.J - j0);
    E* out = g.out;

    if (g.epilogue == EPI_COL_SCATTER) {
        // The tile owns the original columns from its first kept column (0 for the
        // first tile) up to the next tile's first kept column (the full width for
        // the last one).  Thread <-> one aligned pair of original columns.
        for (int q = tid; q < cols_valid; q += NT) idxB[q] = clamp_idx(g.keep[j0 + q], g.out_full);
        __syncthreads();
        const int start = j0 == 0 ? 0 : idxB[0];
        const int end = j0 + BN >= g.J ? g.out_full : clamp_idx(g.keep[j0 + BN], g.out_full);
        for (int pbase = (start & ~1) + 2 * tid; pbase < end; pbase += 2 * NT) {
            const int p0 = pbase, p1 = pbase + 1;
            const bool own0 = p0 >= start, own1 = p1 < end;
            int r0 = lower_bound_lds(idxB, cols_valid, p0);
            const bool k0 = own0 && r0 < cols_valid && idxB[r0] == p0;
            int r1 = r0 + ((r0 < cols_valid && idxB[r0] == p0) ? 1 : 0);
            const bool k1 = own1 && r1 < cols_valid && idxB[r1] == p1;
            r0 = k0 ? r0 : 0;
            r1 = k1 ? r1 : 0;
            E* o = out + (size_t)i0 * (size_t)g.ldo + p0;
            if (own0 && own1) {
                for (int row = 0; row < rows_valid; ++row) {
                    const uint32_t v0 = k0 ? Cs[row * CP + r0] : 0u;
                    const uint32_t v1 = k1 ? Cs[row * CP + r1] : 0u;
                    *(uint32_t*)(o + (size_t)row * (size_t)g.ldo) = v0 | (v1 << 16);
                }
            } else if (own0) {
                for (int row = 0; row < rows_valid; ++row)
                    o[(size_t)row * (size_t)g.ldo] = k0 ? Cs[row * CP + r0] : E(0);
            } else if (own1) {
                for (int row = 0; row < rows_valid; ++row)
                    o[(size_t)row * (size_t)g.ldo + 1] = k1 ? Cs[row * CP + r1] : E(0);
            }
        }
        return;
    }

    const bool scatter_rows = g.epilogue == EPI_ROW_SCATTER;
    if (scatter_rows)
        for (int q = tid; q < rows_valid; q += NT) idxA[q] = clamp_idx(g.keep[i0 + q], g.out_full);
    __syncthreads();
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
        const int end = i0 + BM >= g.I ? g.out_full : clamp_idx(g.keep[i0 + BM], g.out_full);
        for (int p = start + wave; p < end; p += NT / 64) {
            const int ii = lower_bound_lds(idxA, rows_valid, p);
            if (ii < rows_valid && idxA[ii] == p) continue;
            E* o = out + (size_t)p * (size_t)g.ldo + j0;
            for (int j = lane * 8; j < cols_valid; j += 64 * 8) *(uint4*)(o + j) = zero4();
        }
    }
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
template <template <int, int> class LA, template <int, int> class LB, int BM, int BN, int WM, int WN>
int launch_tile(const FArgs& a, hipStream_t stream)
{
    constexpr int smem = fast_smem_bytes<BM, BN>();
    auto fn = fast_kernel<LA, LB, BM, BN, WM, WN>;
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
            return ZR_ERR_HIP;
        attr_set = true;
    }
    FArgs k = a;
    k.tiles_i = (a.I + BM - 1) / BM;
    k.tiles_j = (a.J + BN - 1) / BN;
    const int64_t tiles = (int64_t)k.tiles_i * k.tiles_j;
    const int64_t grid = (tiles + 7) / 8 * 8;
    if (grid > 0x7fffffff) return ZR_ERR_LIMIT;
    hipLaunchKernelGGL(fn, dim3((unsigned)grid), dim3(64 * WM * WN), smem, stream, k);
    return hip_status(hipGetLastError());
}

template <template <int, int> class LA, template <int, int> class LB>
int launch_shape(const FArgs& a, hipStream_t stream)
{
    // tile choice: the largest tile whose grid still fills the 256 CUs reasonably
    const int64_t t256 = (int64_t)((a.I + 255) / 256) * ((a.J + 255) / 256);
    if (t256 >= 200) return launch_tile<LA, LB, 256, 256, 2, 4>(a, stream);
    return launch_tile<LA, LB, 128, 128, 2, 2>(a, stream);
}

}  // namespace

// Returns -1 when the problem is not eligible for this path (the caller then
// uses the general kernel), else a zr_status.
int launch_gemm_fast(const GemmDesc& d, hipStream_t stream)
{
    if (d.dtype != ZR_BF16) return -1;
    auto aligned = [](const void* p, int64_t ld) { return ((uintptr_t)p % 16 == 0) && (ld % 8 == 0); };
    if (!aligned(d.A.base, d.A.ld) || !aligned(d.B.base, d.B.ld) || !aligned(d.out, d.ldo)) return -1;
    // every extent that is walked in 8-element chunks must be a multiple of 8
    auto chunked_ok = [](const Operand& o, int n_rows_canon, int C) {
        if (o.c_contig) {
            if (o.map_contig) return o.map_strided == nullptr && o.n_contig % 2 == 0;   // PG reads aligned dwords
            return C % 8 == 0;                                           // PV: C is the memory row length
        }
        if (o.map_contig) return o.map_strided == nullptr && o.n_contig % 8 == 0;   // QG
        return n_rows_canon % 8 == 0;                                    // QV: J (or I) is the memory row length
    };
    if (!chunked_ok(d.A, d.I, d.C) || !chunked_ok(d.B, d.J, d.C)) return -1;
    if (d.epilogue != EPI_COL_SCATTER && d.J % 8 != 0) return -1;
    if (d.I < 1 || d.J < 1 || d.C < 1) return -1;

    FArgs a;
    a.A = FOp{(const E*)d.A.base, d.A.ld, d.A.map_strided, d.A.map_contig, d.A.n_strided, d.A.n_contig};
    a.B = FOp{(const E*)d.B.base, d.B.ld, d.B.map_strided, d.B.map_contig, d.B.n_strided, d.B.n_contig};
    a.I = d.I; a.J = d.J; a.C = d.C;
    a.out = (E*)d.out; a.ldo = d.ldo; a.epilogue = d.epilogue; a.keep = d.keep_idx; a.out_full = d.out_full;
    a.tiles_i = a.tiles_j = 0;
    const bool ag = d.A.map_contig != nullptr, bg = d.B.map_contig != nullptr;
    if (d.A.c_contig && !d.B.c_contig) {            // forward: A format P, B format Q
        if (!ag && !bg) return launch_shape<LdPV, LdQV>(a, stream);
        if (ag && !bg) return launch_shape<LdPG, LdQV>(a, stream);
        if (!ag && bg) return launch_shape<LdPV, LdQG>(a, stream);
        return -1;
    }
    if (d.A.c_contig && d.B.c_contig) {             // dX: both format P
        if (!ag && !bg) return launch_shape<LdPV, LdPV>(a, stream);
        if (ag && bg) return launch_shape<LdPG, LdPG>(a, stream);
        return -1;
    }
    if (!d.A.c_contig && !d.B.c_contig) {           // dW: both format Q
        if (!ag && !bg) return launch_shape<LdQV, LdQV>(a, stream);
        if (ag && !bg) return launch_shape<LdQG, LdQV>(a, stream);
        if (!ag && bg) return launch_shape<LdQV, LdQG>(a, stream);
        return -1;
    }
    return -1;
}

}  // namespace zr

// Gather-fused MFMA GEMM for the resized shard products (paper Sec. 3.1:
// forward, grad_output and grad_weight of the pruned layer), gfx950 only.
//
// Every product is computed in the canonical form
//     D[i, j] = sum_c A(i, c) * B(j, c)
// on 64-wide wavefronts with the 32x32 MFMA tiles (bf16: 32x32x16, fp32:
// 32x32x2), fp32 accumulation.  The kept-index list is applied while the
// operand tiles travel from HBM into LDS, so no compacted copy of W (or of any
// other operand) ever exists in memory, and the epilogue writes the result at
// its original positions together with the zeros of the dropped positions, so
// the output has its normal shape after one pass (the paper's "recover +
// impute" fused into the product).
//
// LDS tile formats (32-bit words; a bf16 word holds two consecutive
// contraction indices c, c+1 of one row):
//   P  [row][word]  for tensors whose contiguous axis is the contraction axis
//   Q  [word][row]  for tensors whose contiguous axis is the other axis; the
//      two bf16 halves of a word come from two consecutive memory rows, which
//      is what turns the "transposed" operand into MFMA's per-lane k-vectors
//      without any LDS transpose.
// Loader kinds per operand:
//   VEC   16-byte global loads (optionally through a row list: gathers whole
//         rows, e.g. W[S,:])
//   ELEM  element loads through an index list on the contiguous axis (e.g.
//         X[:,S], W[:,S]) - two bf16 loads are packed into one LDS word - and
//         the fallback for unaligned tensors.
#include <cstdio>

#include "zr_common.h"

namespace zr {

namespace {

constexpr int NT = 256;          // threads per workgroup: 4 wavefronts as 2 x 2
constexpr int BKD = 32;          // contraction depth of one LDS tile, in 32-bit words
constexpr int PP = BKD + 4;      // row pitch of format P (words): keeps 16-byte alignment

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int DT> struct Ty;
template <> struct Ty<ZR_BF16> {
    typedef uint16_t E;
    static constexpr int EPD = 2;       // elements per 32-bit word
    static constexpr int DPL = 4;       // words per lane per MFMA
    static constexpr int KDM = 8;       // words of contraction per MFMA (16 elements)
    static constexpr int CPAD = 8;      // C tile pitch padding (elements)
    static __device__ __forceinline__ uint32_t pack(const E* v) { return (uint32_t)v[0] | ((uint32_t)v[1] << 16); }
    static __device__ __forceinline__ E from_f32(float f) { return (E)f32_to_bf16_bits(f); }
    static __device__ __forceinline__ float to_f32(E v) { return bf16_bits_to_f32(v); }
};
template <> struct Ty<ZR_F32> {
    typedef float E;
    static constexpr int EPD = 1;
    static constexpr int DPL = 1;
    static constexpr int KDM = 2;
    static constexpr int CPAD = 4;
    static __device__ __forceinline__ uint32_t pack(const E* v) { return __float_as_uint(v[0]); }
    static __device__ __forceinline__ E from_f32(float f) { return f; }
    static __device__ __forceinline__ float to_f32(E v) { return v; }
};

struct OpView {
    const void* base;
    int64_t ld;
    const int32_t* map_s;   // list on the strided axis or nullptr
    const int32_t* map_c;   // list on the contiguous axis or nullptr
    int n_s, n_c;           // memory extents (for clamping list entries)
};

struct KArgs {
    OpView A, B;
    int I, J, C;
    void* out;
    int64_t ldo;
    int epilogue;
    const int32_t* keep;
    int out_full;
    int out_vec;            // output rows allow 16-byte stores
    int tiles_j;
    const void* prev;       // Same imputation source (layout of out) or nullptr
    int accumulate;         // add the old contents of out (plain epilogue)
    float* avg_partial;     // Average imputation: per-tile sums of the stored results, or nullptr
    int avg_len;            // entries per slot of avg_partial
};

// ---------------------------------------------------------------------------
// Operand loaders.  R = rows of the tile along the operand's non-contraction
// index (BM for A, BN for B).  Each loader keeps one tile in registers
// (fetch) and later writes it to LDS (commit), so the global loads of tile
// k+1 overlap the MFMAs of tile k.
// ---------------------------------------------------------------------------

// Format P, vector loads: 8 chunks of 4 words per row.
template <int DT, int R>
struct LoadPVec {
    typedef typename Ty<DT>::E E;
    static constexpr int EPD = Ty<DT>::EPD;
    static constexpr int N = R / 32;            // chunks per thread
    static constexpr int LDS_WORDS = R * PP;
    const E* rowptr[N];
    uint4 v[N];

    __device__ __forceinline__ void init(const OpView& op, int r0, int rlim, int tid)
    {
#pragma unroll
        for (int it = 0; it < N; ++it) {
            const int row = (tid + NT * it) >> 3;
            const int i = r0 + row;
            if (i < rlim) {
                const int srow = op.map_s ? clamp_idx(op.map_s[i], op.n_s) : i;
                rowptr[it] = (const E*)op.base + (size_t)srow * (size_t)op.ld;
            } else {
                rowptr[it] = nullptr;
            }
        }
    }
    __device__ __forceinline__ void fetch(const OpView&, int c0, int C, int tid)
    {
#pragma unroll
        for (int it = 0; it < N; ++it) {
            const int ch = (tid + NT * it) & 7;
            const int c = c0 + ch * 4 * EPD;
            uint4 val = make_uint4(0, 0, 0, 0);
            if (rowptr[it] != nullptr && c < C) {
                if (c + 4 * EPD <= C) {
                    val = *(const uint4*)(rowptr[it] + c);
                } else {
                    uint32_t w[4];
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        E e[2] = {E(0), E(0)};
#pragma unroll
                        for (int q = 0; q < EPD; ++q) {
                            const int cc = c + d * EPD + q;
                            if (cc < C) e[q] = rowptr[it][cc];
                        }
                        w[d] = Ty<DT>::pack(e);
                    }
                    val = make_uint4(w[0], w[1], w[2], w[3]);
                }
            }
            v[it] = val;
        }
    }
    __device__ __forceinline__ void commit(uint32_t* lds, int tid) const
    {
#pragma unroll
        for (int it = 0; it < N; ++it) {
            const int q = tid + NT * it;
            *(uint4*)(lds + (q >> 3) * PP + (q & 7) * 4) = v[it];
        }
    }
};

// Format P, element loads through optional lists on both axes.
template <int DT, int R>
struct LoadPElem {
    typedef typename Ty<DT>::E E;
    static constexpr int EPD = Ty<DT>::EPD;
    static constexpr int N = R / 8;             // words per thread
    static constexpr int LDS_WORDS = R * PP;
    int r0_, rlim_;
    uint32_t v[N];

    __device__ __forceinline__ void init(const OpView&, int r0, int rlim, int) { r0_ = r0; rlim_ = rlim; }
    __device__ __forceinline__ void fetch(const OpView& op, int c0, int C, int tid)
    {
        const int kd = tid & 31;
        int col[2];
        bool ok[2];
#pragma unroll
        for (int q = 0; q < EPD; ++q) {
            const int c = c0 + kd * EPD + q;
            ok[q] = c < C;
            col[q] = 0;
            if (ok[q]) col[q] = op.map_c ? clamp_idx(op.map_c[c], op.n_c) : c;
        }
#pragma unroll
        for (int it = 0; it < N; ++it) {
            const int i = r0_ + (tid >> 5) + 8 * it;
            E e[2] = {E(0), E(0)};
            if (i < rlim_) {
                const int srow = op.map_s ? clamp_idx(op.map_s[i], op.n_s) : i;
                const E* p = (const E*)op.base + (size_t)srow * (size_t)op.ld;
#pragma unroll
                for (int q = 0; q < EPD; ++q)
                    if (ok[q]) e[q] = p[col[q]];
            }
            v[it] = Ty<DT>::pack(e);
        }
    }
    __device__ __forceinline__ void commit(uint32_t* lds, int tid) const
    {
#pragma unroll
        for (int it = 0; it < N; ++it)
            lds[((tid >> 5) + 8 * it) * PP + (tid & 31)] = v[it];
    }
};

// Format Q, vector loads.  bf16: a unit is 8 rows-of-the-tile x 2 memory rows
// (c, c+1), interleaved into 8 words.  fp32: a unit is 4 words of one memory row.
template <int DT, int R>
struct LoadQVec {
    typedef typename Ty<DT>::E E;
    static constexpr int EPD = Ty<DT>::EPD;
    static constexpr int PQ = R + 8;
    static constexpr int LDS_WORDS = BKD * PQ;
    static constexpr int JCH = (DT == ZR_BF16) ? 8 : 4;        // tile rows per unit
    static constexpr int UPR = R / JCH;                         // units per word-row
    static constexpr int N = BKD * UPR / NT;                    // units per thread
    int r0_, rlim_;
    uint4 lo[N];
    uint4 hi[(DT == ZR_BF16) ? N : 1];

    __device__ __forceinline__ void init(const OpView&, int r0, int rlim, int) { r0_ = r0; rlim_ = rlim; }

    __device__ __forceinline__ uint4 load_row(const OpView& op, int c, int C, int j) const
    {
        uint4 val = make_uint4(0, 0, 0, 0);
        if (c < C && j < rlim_) {
            const int srow = op.map_s ? clamp_idx(op.map_s[c], op.n_s) : c;
            const E* p = (const E*)op.base + (size_t)srow * (size_t)op.ld + j;
            if (j + JCH <= rlim_) {
                val = *(const uint4*)p;
            } else {
                E e[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) e[q] = (q < JCH && j + q < rlim_) ? p[q] : E(0);
                if constexpr (DT == ZR_BF16)
                    val = make_uint4(Ty<DT>::pack(e), Ty<DT>::pack(e + 2), Ty<DT>::pack(e + 4), Ty<DT>::pack(e + 6));
                else
                    val = make_uint4(Ty<DT>::pack(e), Ty<DT>::pack(e + 1), Ty<DT>::pack(e + 2), Ty<DT>::pack(e + 3));
            }
        }
        return val;
    }
    __device__ __forceinline__ void fetch(const OpView& op, int c0, int C, int tid)
    {
#pragma unroll
        for (int it = 0; it < N; ++it) {
            const int q = tid + NT * it;
            const int kd = q / UPR;
            const int j = r0_ + (q % UPR) * JCH;
            if constexpr (DT == ZR_BF16) {
                lo[it] = load_row(op, c0 + 2 * kd, C, j);
                hi[it] = load_row(op, c0 + 2 * kd + 1, C, j);
            } else {
                lo[it] = load_row(op, c0 + kd, C, j);
            }
        }
    }
    __device__ __forceinline__ void commit(uint32_t* lds, int tid) const
    {
#pragma unroll
        for (int it = 0; it < N; ++it) {
            const int q = tid + NT * it;
            uint32_t* dst = lds + (q / UPR) * PQ + (q % UPR) * JCH;
            if constexpr (DT == ZR_BF16) {
                const uint32_t a[4] = {lo[it].x, lo[it].y, lo[it].z, lo[it].w};
                const uint32_t b[4] = {hi[it].x, hi[it].y, hi[it].z, hi[it].w};
                uint32_t w[8];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    w[2 * t] = (a[t] & 0xffffu) | (b[t] << 16);
                    w[2 * t + 1] = (a[t] >> 16) | (b[t] & 0xffff0000u);
                }
                *(uint4*)dst = make_uint4(w[0], w[1], w[2], w[3]);
                *(uint4*)(dst + 4) = make_uint4(w[4], w[5], w[6], w[7]);
            } else {
                *(uint4*)dst = lo[it];
            }
        }
    }
};

// Format Q, element loads: thread <-> one tile row j (its memory column is
// looked up once per tile), looping over the words of the contraction tile.
template <int DT, int R>
struct LoadQElem {
    typedef typename Ty<DT>::E E;
    static constexpr int EPD = Ty<DT>::EPD;
    static constexpr int PQ = R + 8;
    static constexpr int LDS_WORDS = BKD * PQ;
    static constexpr int N = R / 8;             // words per thread
    static constexpr int KSTEP = NT / R > 0 ? NT / R : 1;
    static_assert(R <= NT, "tile rows beyond the thread count are not laid out");
    int col_;
    bool okj_;
    uint32_t v[N];

    __device__ __forceinline__ void init(const OpView& op, int r0, int rlim, int tid)
    {
        const int j = r0 + (tid % R);
        okj_ = j < rlim;
        col_ = 0;
        if (okj_) col_ = op.map_c ? clamp_idx(op.map_c[j], op.n_c) : j;
    }
    __device__ __forceinline__ void fetch(const OpView& op, int c0, int C, int tid)
    {
#pragma unroll
        for (int it = 0; it < N; ++it) {
            const int kd = tid / R + KSTEP * it;
            E e[2] = {E(0), E(0)};
#pragma unroll
            for (int q = 0; q < EPD; ++q) {
                const int c = c0 + kd * EPD + q;
                if (okj_ && c < C) {
                    const int srow = op.map_s ? clamp_idx(op.map_s[c], op.n_s) : c;
                    e[q] = ((const E*)op.base)[(size_t)srow * (size_t)op.ld + col_];
                }
            }
            v[it] = Ty<DT>::pack(e);
        }
    }
    __device__ __forceinline__ void commit(uint32_t* lds, int tid) const
    {
#pragma unroll
        for (int it = 0; it < N; ++it)
            lds[(tid / R + KSTEP * it) * PQ + (tid % R)] = v[it];
    }
};

template <int DT, bool CC, bool VEC, int R> struct PickLoader;
template <int DT, int R> struct PickLoader<DT, true, true, R> { typedef LoadPVec<DT, R> type; };
template <int DT, int R> struct PickLoader<DT, true, false, R> { typedef LoadPElem<DT, R> type; };
template <int DT, int R> struct PickLoader<DT, false, true, R> { typedef LoadQVec<DT, R> type; };
template <int DT, int R> struct PickLoader<DT, false, false, R> { typedef LoadQElem<DT, R> type; };

// ---------------------------------------------------------------------------
// MFMA fragment reads
// ---------------------------------------------------------------------------
template <int DT, bool CC, int R> struct Frag;

template <bool CC, int R> struct Frag<ZR_BF16, CC, R> {
    typedef bf16x8 type;
    // row: tile row of this lane; kd: first word of this lane's 4-word k-vector
    static __device__ __forceinline__ type read(const uint32_t* lds, int row, int kd)
    {
        union { uint4 u; bf16x8 b; } x;
        if (CC) {
            x.u = *(const uint4*)(lds + row * PP + kd);
        } else {
            constexpr int PQ = R + 8;
            x.u = make_uint4(lds[kd * PQ + row], lds[(kd + 1) * PQ + row],
                             lds[(kd + 2) * PQ + row], lds[(kd + 3) * PQ + row]);
        }
        return x.b;
    }
};
template <bool CC, int R> struct Frag<ZR_F32, CC, R> {
    typedef float type;
    static __device__ __forceinline__ type read(const uint32_t* lds, int row, int kd)
    {
        constexpr int PQ = R + 8;
        return __uint_as_float(CC ? lds[row * PP + kd] : lds[kd * PQ + row]);
    }
};

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mfma(float a, float b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// first position in the ascending LDS list s[0..n) with s[pos] >= p
__device__ __forceinline__ int lower_bound_lds(const int* s, int n, int p)
{
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (s[mid] < p) lo = mid + 1; else hi = mid;
    }
    return lo;
}

template <int BM, int BN, int DT>
constexpr int smem_bytes()
{
    // operand stages: the larger of the two formats for each operand, two stages
    constexpr int a_words = BM * PP > BKD * (BM + 8) ? BM * PP : BKD * (BM + 8);
    constexpr int b_words = BN * PP > BKD * (BN + 8) ? BN * PP : BKD * (BN + 8);
    constexpr int stage_bytes = 2 * (a_words + b_words) * 4;
    // epilogue: C tile in the output type plus the index tile
    constexpr int esz = DT == ZR_BF16 ? 2 : 4;
    constexpr int c_bytes = BM * (BN + Ty<DT>::CPAD) * esz + (BM > BN ? BM : BN) * 4;
    return stage_bytes > c_bytes ? stage_bytes : c_bytes;
}

// ---------------------------------------------------------------------------
// The kernel
// ---------------------------------------------------------------------------
template <int DT, bool ACC, bool AVEC, bool BCC, bool BVEC, int BM, int BN>
__global__ __launch_bounds__(NT) void gemm_kernel(const KArgs g)
{
    typedef typename Ty<DT>::E E;
    constexpr int DPL = Ty<DT>::DPL;
    constexpr int KDM = Ty<DT>::KDM;
    constexpr int EPD = Ty<DT>::EPD;
    constexpr int TM = BM / 64, TN = BN / 64;          // 32x32 tiles per wavefront
    constexpr int A_WORDS = BM * PP > BKD * (BM + 8) ? BM * PP : BKD * (BM + 8);
    constexpr int B_WORDS = BN * PP > BKD * (BN + 8) ? BN * PP : BKD * (BN + 8);
    constexpr int CP = BN + Ty<DT>::CPAD;
    typedef typename PickLoader<DT, ACC, AVEC, BM>::type LA;
    typedef typename PickLoader<DT, BCC, BVEC, BN>::type LB;

    extern __shared__ __align__(16) uint32_t smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l32 = lane & 31;
    const int grp = lane >> 5;
    const int wr0 = (wave >> 1) * (BM / 2);
    const int wc0 = (wave & 1) * (BN / 2);

    const int ti = blockIdx.x / g.tiles_j;
    const int tj = blockIdx.x % g.tiles_j;
    const int i0 = ti * BM, j0 = tj * BN;

    constexpr int STAGE_WORDS = A_WORDS + B_WORDS;   // stage s: A tile, then B tile

    f32x16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
    if (g.accumulate) {
        // the accumulators start from the old contents of the output (one rounding
        // at the end); done here, where no other registers are live yet
        const int rows_in_tile = min(BM, g.I - i0), cols_in_tile = min(BN, g.J - j0);
        const E* old = (const E*)g.out;
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    // coordinates clamped into the tile instead of a guard: the loads need no
                    // branches and go out together; accumulators outside the tile are never stored
                    const int row = min(wr0 + a * 32 + (r >> 2) * 8 + grp * 4 + (r & 3), rows_in_tile - 1);
                    const int col = min(wc0 + b * 32 + l32, cols_in_tile - 1);
                    acc[a][b][r] = Ty<DT>::to_f32(old[(size_t)(i0 + row) * (size_t)g.ldo + j0 + col]);
                }
    }

    LA la;
    LB lb;
    la.init(g.A, i0, g.I, tid);
    lb.init(g.B, j0, g.J, tid);

    const int KT = (g.C + BKD * EPD - 1) / (BKD * EPD);
    la.fetch(g.A, 0, g.C, tid);
    lb.fetch(g.B, 0, g.C, tid);
    la.commit(smem, tid);
    lb.commit(smem + A_WORDS, tid);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < KT;
        if (more) {
            la.fetch(g.A, (kt + 1) * BKD * EPD, g.C, tid);
            lb.fetch(g.B, (kt + 1) * BKD * EPD, g.C, tid);
        }
        const uint32_t* as = smem + cur * STAGE_WORDS;
        const uint32_t* bs = as + A_WORDS;
#pragma unroll
        for (int step = 0; step < BKD / KDM; ++step) {
            const int kd = step * KDM + grp * DPL;
            typename Frag<DT, ACC, BM>::type af[TM];
            typename Frag<DT, BCC, BN>::type bf[TN];
#pragma unroll
            for (int a = 0; a < TM; ++a) af[a] = Frag<DT, ACC, BM>::read(as, wr0 + a * 32 + l32, kd);
#pragma unroll
            for (int b = 0; b < TN; ++b) bf[b] = Frag<DT, BCC, BN>::read(bs, wc0 + b * 32 + l32, kd);
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b) acc[a][b] = mfma(af[a], bf[b], acc[a][b]);
        }
        if (more) {
            la.commit(smem + (cur ^ 1) * STAGE_WORDS, tid);
            lb.commit(smem + (cur ^ 1) * STAGE_WORDS + A_WORDS, tid);
        }
        __syncthreads();
    }

    // ---- epilogue: accumulators -> C tile in LDS (output type) ---------------
    E* Cs = (E*)smem;
    int* sidx = (int*)(Cs + BM * CP);
    const int rows_valid = min(BM, g.I - i0);
    const int cols_valid = min(BN, g.J - j0);
    E* out = (E*)g.out;
    const E* prev = (const E*)g.prev;
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = wr0 + a * 32 + (r >> 2) * 8 + grp * 4 + (r & 3);
                Cs[row * CP + wc0 + b * 32 + l32] = Ty<DT>::from_f32(acc[a][b][r]);
            }
    constexpr int VEC = 16 / (int)sizeof(E);

    if (g.epilogue == EPI_COL_SCATTER) {
        // this tile owns the original columns from its first kept column (0 for
        // the first tile) up to the next tile's first kept column (the full
        // width for the last tile); kept ones receive results, the rest +0
        for (int q = tid; q < cols_valid; q += NT) sidx[q] = clamp_idx(g.keep[j0 + q], g.out_full);
        __syncthreads();
        if (g.avg_partial) {
            // sum of this tile's stored (rounded) results per output row, in column order
            float* dst = g.avg_partial + (size_t)tj * (size_t)g.avg_len + i0;
            for (int row = tid; row < rows_valid; row += NT) {
                float sum = 0.f;
                for (int c = 0; c < cols_valid; ++c) sum += Ty<DT>::to_f32(Cs[row * CP + c]);
                dst[row] = sum;
            }
        }
        const int start = j0 == 0 ? 0 : sidx[0];
        const int end = j0 + BN >= g.J ? g.out_full : clamp_idx(g.keep[j0 + BN], g.out_full);
        for (int chunk = start; chunk < end; chunk += NT) {
            const int p = chunk + tid;
            if (p < end) {
                const int jj = lower_bound_lds(sidx, cols_valid, p);
                const bool hit = jj < cols_valid && sidx[jj] == p;
                E* o = out + (size_t)i0 * (size_t)g.ldo + p;
                if (hit || !prev) {
                    for (int row = 0; row < rows_valid; ++row)
                        o[(size_t)row * (size_t)g.ldo] = hit ? Cs[row * CP + jj] : E(0);
                } else {
                    // Same: a position is read and written by this thread only (also when the
                    // previous tensor is the output itself), so loads go out in batches
                    const E* pv = prev + (size_t)i0 * (size_t)g.ldo + p;
                    constexpr int RB = 16;
                    for (int row = 0; row < rows_valid; row += RB) {
                        E old[RB];
#pragma unroll
                        for (int u = 0; u < RB; ++u)
                            old[u] = row + u < rows_valid ? pv[(size_t)(row + u) * (size_t)g.ldo] : E(0);
#pragma unroll
                        for (int u = 0; u < RB; ++u) {
                            if (row + u >= rows_valid) break;
                            o[(size_t)(row + u) * (size_t)g.ldo] = old[u];
                        }
                    }
                }
            }
        }
        return;
    }

    const bool scatter_rows = g.epilogue == EPI_ROW_SCATTER;
    if (scatter_rows) {
        for (int q = tid; q < rows_valid; q += NT) sidx[q] = clamp_idx(g.keep[i0 + q], g.out_full);
    }
    __syncthreads();
    if (scatter_rows && g.avg_partial) {
        // sum of this tile's stored (rounded) results per output column, in row order
        float* dst = g.avg_partial + (size_t)ti * (size_t)g.avg_len + j0;
        for (int col = tid; col < cols_valid; col += NT) {
            float sum = 0.f;
            for (int r = 0; r < rows_valid; ++r) sum += Ty<DT>::to_f32(Cs[r * CP + col]);
            dst[col] = sum;
        }
    }
    constexpr int CPR = BN / VEC;               // 16-byte chunks per tile row
    for (int q = tid; q < BM * CPR; q += NT) {
        const int row = q / CPR;
        const int j = (q % CPR) * VEC;
        if (row >= rows_valid || j >= cols_valid) continue;
        const int orow = scatter_rows ? sidx[row] : i0 + row;
        E* o = out + (size_t)orow * (size_t)g.ldo + j0 + j;
        const E* c = Cs + row * CP + j;
        if (g.out_vec && j + VEC <= cols_valid) {
            *(uint4*)o = *(const uint4*)c;
        } else {
            for (int t = 0; t < VEC && j + t < cols_valid; ++t) o[t] = c[t];
        }
    }
    if (scatter_rows) {
        // zero the dropped rows this tile owns (same ownership rule as above)
        const int start = i0 == 0 ? 0 : sidx[0];
        const int end = i0 + BM >= g.I ? g.out_full : clamp_idx(g.keep[i0 + BM], g.out_full);
        // every lane looks one row up, the wavefront then writes the dropped ones together
        for (int base = start + wave * 64; base < end; base += NT) {
            const int mine = base + lane;
            bool dropped = false;
            if (mine < end) {
                const int ii = lower_bound_lds(sidx, rows_valid, mine);
                dropped = !(ii < rows_valid && sidx[ii] == mine);
            }
            unsigned long long todo = __ballot(dropped);
            while (todo) {
                const int p = base + (__ffsll((long long)todo) - 1);
                todo &= todo - 1;
                E* o = out + (size_t)p * (size_t)g.ldo + j0;
                const E* pv = prev ? prev + (size_t)p * (size_t)g.ldo + j0 : nullptr;
                for (int j = lane; j < cols_valid; j += 64) o[j] = pv ? pv[j] : E(0);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
template <int DT, bool ACC, bool AVEC, bool BCC, bool BVEC, int BM, int BN>
int launch_inst(const KArgs& k, hipStream_t stream)
{
    constexpr int smem = smem_bytes<BM, BN, DT>();
    auto fn = gemm_kernel<DT, ACC, AVEC, BCC, BVEC, BM, BN>;
    static AttrFlags attr_set;      // per instantiation and device
    if (!ensure_max_dynamic_lds((const void*)fn, smem, &attr_set)) return ZR_ERR_HIP;
    if (debug_names_wanted())
        snprintf(g_debug.last_kernel, sizeof(g_debug.last_kernel), "gemm_kernel<%d, %s, %s, %s, %s, %d, %d>", DT,
                 ACC ? "true" : "false", AVEC ? "true" : "false", BCC ? "true" : "false", BVEC ? "true" : "false", BM, BN);
    KArgs kk = k;
    kk.tiles_j = (k.J + BN - 1) / BN;
    const int64_t tiles = (int64_t)((k.I + BM - 1) / BM) * kk.tiles_j;
    if (tiles > 0x7fffffff) return ZR_ERR_LIMIT;
    hipLaunchKernelGGL(fn, dim3((unsigned)tiles), dim3(NT), smem, stream, kk);
    return hip_status(hipGetLastError());
}

template <int DT, bool ACC, bool BCC>
int launch_fmt(const KArgs& k, bool avec, bool bvec, hipStream_t stream)
{
    constexpr int BM = 128, BN = 128;
    if (avec && bvec) return launch_inst<DT, ACC, true, BCC, true, BM, BN>(k, stream);
    if (avec) return launch_inst<DT, ACC, true, BCC, false, BM, BN>(k, stream);
    if (bvec) return launch_inst<DT, ACC, false, BCC, true, BM, BN>(k, stream);
    return launch_inst<DT, ACC, false, BCC, false, BM, BN>(k, stream);
}

template <int DT>
int launch_dt(const GemmDesc& d, hipStream_t stream)
{
    constexpr int esz = DT == ZR_BF16 ? 2 : 4;
    constexpr int VEC = 16 / esz;
    auto vec_ok = [&](const Operand& o) {
        return o.map_contig == nullptr && ((uintptr_t)o.base % 16 == 0) && (o.ld % VEC == 0);
    };
    KArgs k;
    k.A = OpView{d.A.base, d.A.ld, d.A.map_strided, d.A.map_contig, d.A.n_strided, d.A.n_contig};
    k.B = OpView{d.B.base, d.B.ld, d.B.map_strided, d.B.map_contig, d.B.n_strided, d.B.n_contig};
    k.I = d.I; k.J = d.J; k.C = d.C;
    k.out = d.out; k.ldo = d.ldo; k.epilogue = d.epilogue; k.keep = d.keep_idx; k.out_full = d.out_full;
    k.out_vec = ((uintptr_t)d.out % 16 == 0) && (d.ldo % VEC == 0);
    k.tiles_j = 0;
    k.prev = d.prev; k.accumulate = d.accumulate ? 1 : 0;
    k.avg_partial = d.epilogue == EPI_PLAIN ? nullptr : d.avg_partial; k.avg_len = d.avg_len;
    const bool av = vec_ok(d.A), bv = vec_ok(d.B);
    if (d.A.c_contig && !d.B.c_contig) return launch_fmt<DT, true, false>(k, av, bv, stream);
    if (d.A.c_contig && d.B.c_contig) return launch_fmt<DT, true, true>(k, av, bv, stream);
    if (!d.A.c_contig && !d.B.c_contig) return launch_fmt<DT, false, false>(k, av, bv, stream);
    return ZR_ERR_MODE;
}

}  // namespace

thread_local DebugState g_debug;

bool ensure_max_dynamic_lds(const void* fn, int bytes, void* flags16)
{
    AttrFlags* f = (AttrFlags*)flags16;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    if (dev < 0 || dev >= AttrFlags::MAX_DEVICES) {      // beyond the table: set it every time
        return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) == hipSuccess;
    }
    if (f->done[dev].load(std::memory_order_acquire)) return true;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return false;
    f->done[dev].store(true, std::memory_order_release);
    return true;
}

static int launch_gemm_untimed(const GemmDesc& d, hipStream_t stream)
{
    const int fast = launch_gemm_fast(d, stream);   // bf16, 16-byte aligned rows
    if (fast >= 0) return fast;
    if (d.dtype == ZR_BF16) return launch_dt<ZR_BF16>(d, stream);
    if (d.dtype == ZR_F32) return launch_dt<ZR_F32>(d, stream);
    return ZR_ERR_DTYPE;
}

int launch_gemm(const GemmDesc& d, hipStream_t stream)
{
    if (!g_debug.armed_once) return launch_gemm_untimed(d, stream);
    // measuring aid (zr_debug_time_next_product): events right around this product's own
    // launch(es), without a preceding extraction or a following imputation pass.  One shot.
    hipEvent_t e0 = g_debug.start, e1 = g_debug.stop;
    if (hipEventRecord(e0, stream) != hipSuccess) { g_debug.armed_once = false; return ZR_ERR_HIP; }
    const int st = launch_gemm_untimed(d, stream);
    g_debug.armed_once = false;
    g_debug.start = g_debug.stop = nullptr;
    if (hipEventRecord(e1, stream) != hipSuccess) return ZR_ERR_HIP;
    return st;
}

}  // namespace zr

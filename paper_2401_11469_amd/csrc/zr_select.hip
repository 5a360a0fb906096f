// Priority selection: the n' highest-score indices, emitted ascending
// (Algorithm 1 of the paper: top-L_pri select, then ascending sort), plus the
// complementary pruned set P of the lineage tuple (Sec. 3.1).
//
// No sort is needed: a 4-pass MSB radix select finds the n'-th largest order
// key T and how many keys are strictly greater; one ordered pass over the
// indices then keeps every index whose key is > T and the first (by index) of
// those equal to T, writing kept and pruned indices by prefix position, which
// makes both lists ascending by construction.
//
// One workgroup per score vector: 1024 threads (16 wavefronts of 64) for a single
// vector, where latency is what counts, 256 threads when many vectors are
// selected in one launch, so that 8 of them share a compute unit and the chip's
// memory system stays busy.  Vectors of up to 12288 scores are turned into order
// keys once and kept in LDS (sized to the vector), so the five passes read HBM a
// single time; longer ones re-read from memory.
#include "zr_common.h"

namespace zr {

namespace {

constexpr int SEL_THREADS = 1024;      // single vector
constexpr int SEL_THREADS_MANY = 256;  // many vectors per launch

// Monotone map fp32 -> uint32: larger score <=> larger key.  NaN -> 0 (lowest,
// below -inf); -0.0 and +0.0 share one key.
__device__ __forceinline__ uint32_t order_key(float s)
{
    uint32_t u = __float_as_uint(s);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;   // NaN
    if ((u & 0x7fffffffu) == 0u) u = 0u;              // -0.0 -> +0.0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr int SEL_LDS_KEYS = 12288;    // 48 KB of order keys

// One workgroup selects one score vector s[n]: keep[n_keep] and drop[n - n_keep].
template <bool STAGED, int NT>
__device__ __forceinline__ void select_body(const float* __restrict__ s, int n, int n_keep,
                                            int32_t* __restrict__ keep, int32_t* __restrict__ drop)
{
    constexpr int SEL_WAVES = NT / 64;
    static_assert(NT >= 256 && NT % 64 == 0, "the histogram is cleared by the first 256 threads");
    extern __shared__ uint32_t keys[];            // n order keys when STAGED (dynamic size)
    __shared__ uint32_t hist[256];
    __shared__ uint32_t s_digit, s_remaining;
    __shared__ uint32_t wave_gt[SEL_WAVES], wave_eq[SEL_WAVES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;

    if (STAGED) {
        for (int i = tid; i < n; i += NT) keys[i] = order_key(s[i]);
        __syncthreads();
    }
    auto key_at = [&](int i) -> uint32_t { return STAGED ? keys[i] : order_key(s[i]); };

    // ---- radix select of the n_keep-th largest key -------------------------
    uint32_t prefix = 0, mask = 0, remaining = (uint32_t)n_keep;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (int i = tid; i < n; i += NT) {
            const uint32_t k = key_at(i);
            if ((k & mask) == prefix) atomicAdd(&hist[(k >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (wave == 0) {
            // lane l owns bins 4l..4l+3; suffix sums give, for each bin, the
            // number of candidates in strictly higher bins
            uint32_t h[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) h[q] = hist[4 * lane + q];
            const uint32_t mine = h[0] + h[1] + h[2] + h[3];
            uint32_t incl = mine;                       // inclusive suffix sum over lanes
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t v = __shfl_down(incl, off, 64);
                if (lane + off < 64) incl += v;
            }
            uint32_t above = incl - mine;               // candidates in lanes > this one
#pragma unroll
            for (int q = 3; q >= 0; --q) {
                if (above < remaining && remaining <= above + h[q]) {
                    s_digit = (uint32_t)(4 * lane + q);
                    s_remaining = remaining - above;
                }
                above += h[q];
            }
        }
        __syncthreads();
        prefix |= s_digit << shift;
        mask |= 0xffu << shift;
        remaining = s_remaining;
        __syncthreads();
    }
    const uint32_t T = prefix;          // the n_keep-th largest key
    const uint32_t need_eq = remaining; // how many of the keys == T are kept (>= 1)

    // ---- ordered compaction -----------------------------------------------
    uint32_t run_gt = 0, run_eq = 0;    // totals over all earlier chunks
    for (int base = 0; base < n; base += NT) {
        const int i = base + tid;
        bool gt = false, eq = false;
        if (i < n) {
            const uint32_t k = key_at(i);
            gt = k > T;
            eq = k == T;
        }
        const uint64_t bgt = __ballot(gt);
        const uint64_t beq = __ballot(eq);
        const uint64_t below = (1ull << lane) - 1ull;
        if (lane == 0) {
            wave_gt[wave] = (uint32_t)__popcll(bgt);
            wave_eq[wave] = (uint32_t)__popcll(beq);
        }
        __syncthreads();
        uint32_t pre_gt = run_gt + (uint32_t)__popcll(bgt & below);
        uint32_t pre_eq = run_eq + (uint32_t)__popcll(beq & below);
        uint32_t tot_gt = 0, tot_eq = 0;
#pragma unroll
        for (int w = 0; w < SEL_WAVES; ++w) {
            const uint32_t g = wave_gt[w], e = wave_eq[w];
            if (w < wave) { pre_gt += g; pre_eq += e; }
            tot_gt += g;
            tot_eq += e;
        }
        if (i < n) {
            const bool kept = gt || (eq && pre_eq < need_eq);
            // kept indices before i: all greater ones plus the first need_eq equal ones
            const uint32_t kept_before = pre_gt + (pre_eq < need_eq ? pre_eq : need_eq);
            // positions are in range by construction; the comparisons only make
            // an out-of-range store impossible whatever the scores hold
            if (kept) {
                if (kept_before < (uint32_t)n_keep) keep[kept_before] = i;
            } else if (drop) {
                const uint32_t pos = (uint32_t)i - kept_before;
                if (pos < (uint32_t)(n - n_keep)) drop[pos] = i;
            }
        }
        run_gt += tot_gt;
        run_eq += tot_eq;
        __syncthreads();
    }
}

template <bool STAGED, int NT>
__global__ __launch_bounds__(NT) void select_kernel(
    const float* __restrict__ scores, int n, int n_keep,
    int32_t* __restrict__ keep_idx, int32_t* __restrict__ drop_idx, int64_t ld_idx)
{
    select_body<STAGED, NT>(scores + (size_t)blockIdx.x * (size_t)n, n, n_keep,
                        keep_idx + (size_t)blockIdx.x * (size_t)ld_idx,
                        drop_idx ? drop_idx + (size_t)blockIdx.x * (size_t)ld_idx : nullptr);
}

// Several vectors of different lengths in one launch (the projections of a layer
// shard): workgroup b takes descriptor b.  The descriptors travel as a kernel
// argument, no device memory is involved.
template <bool STAGED>
__global__ __launch_bounds__(SEL_THREADS) void select_multi_kernel(const SelectMulti m)
{
    const int b = blockIdx.x;
    select_body<STAGED, SEL_THREADS>(m.scores[b], m.n[b], m.n_keep[b], m.keep[b], m.drop[b]);
}

// ---------------------------------------------------------------------------
// One long vector on many workgroups (with scratch from the caller).  The same
// selection as select_body, cut into launches; every launch reads the vector once:
//   clear     the four global histograms
//   hist p    (p = 0..3) each workgroup histograms digit p of the keys of its slice that
//             match the digits chosen so far (which every wavefront first derives again
//             from the global histograms of the passes before: 256 counters per pass),
//             in LDS, then adds its 256 counters to the global histogram of the pass
//   count     the last digit gives T and how many keys equal to T are kept; each
//             WAVEFRONT counts the keys > T and == T of its 4096 scores
//   scan      one workgroup: exclusive prefix sums of those counts over the wavefronts
//   write     the ordered pass, each wavefront on its own 4096 scores with no barrier:
//             position = the wavefront's prefix + the position inside it
// All counters are integers (order-free); the lists are the same, bit for bit, as
// those of the single-workgroup kernel.
// Scratch (uint32 words): [0, 1024) histograms; [1024, 1032) T, kept-equal count;
// then gt count, eq count, gt prefix, eq prefix: 4 x WIDE_MAX_GROUPS.
// ---------------------------------------------------------------------------
constexpr int WIDE_THREADS = 256;
constexpr int WIDE_WAVE_SLICE = 4096;                          // scores per wavefront
constexpr int WIDE_SLICE = WIDE_WAVE_SLICE * (WIDE_THREADS / 64);   // per workgroup (64 KB)
constexpr int WIDE_MAX_GROUPS = (1 << 24) / WIDE_WAVE_SLICE;   // 4096 wavefronts: the longest vector the entry points take
constexpr int WIDE_STATE = 1024;
constexpr int WIDE_COUNTS = 1032;
constexpr size_t WIDE_WORDS = WIDE_COUNTS + 4 * (size_t)WIDE_MAX_GROUPS;
constexpr int WIDE_COPIES = 8;                                 // copies of the LDS histogram

// A wavefront picks the digit of one pass from its 256 counters: the bin that holds the
// `remaining`-th largest candidate (bins taken from the top), and how many candidates of that
// bin are still wanted.  Every lane returns the result.
__device__ __forceinline__ void wide_pick(const uint32_t* __restrict__ h256, uint32_t remaining, int lane,
                                          uint32_t& digit, uint32_t& remaining_out)
{
    uint32_t h[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) h[q] = h256[4 * lane + q];
    const uint32_t mine = h[0] + h[1] + h[2] + h[3];
    uint32_t incl = mine;                       // inclusive suffix sum over lanes
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t v = __shfl_down(incl, off, 64);
        if (lane + off < 64) incl += v;
    }
    uint32_t above = incl - mine;
    uint32_t d = 0xffffffffu, r = 0;
#pragma unroll
    for (int q = 3; q >= 0; --q) {
        if (above < remaining && remaining <= above + h[q]) { d = (uint32_t)(4 * lane + q); r = remaining - above; }
        above += h[q];
    }
    // exactly one lane found it
    const uint64_t who = __ballot(d != 0xffffffffu);
    const int src = who ? (int)(__ffsll((long long)who) - 1) : 0;
    digit = __shfl(d, src, 64);
    remaining_out = __shfl(r, src, 64);
}

// prefix / mask / remaining after the first `passes` digits, from the global histograms
// (run by every wavefront for itself: no LDS, no barrier)
__device__ __forceinline__ void wide_replay(const uint32_t* __restrict__ ghist, int passes, uint32_t n_keep, int lane,
                                            uint32_t& prefix, uint32_t& mask, uint32_t& remaining)
{
    prefix = 0; mask = 0; remaining = n_keep;
    for (int p = 0; p < passes; ++p) {
        uint32_t digit, rem;
        wide_pick(ghist + 256 * p, remaining, lane, digit, rem);
        const int shift = 24 - 8 * p;
        prefix |= digit << shift;
        mask |= 0xffu << shift;
        remaining = rem;
    }
}

__global__ __launch_bounds__(1024) void wide_clear_kernel(uint32_t* __restrict__ ws)
{
    if (threadIdx.x < 1024) ws[threadIdx.x] = 0;
}

// One workgroup of 1024 threads per compute unit, each on a contiguous share of the vector: with
// one workgroup per 16384 scores the 256 global counters of a pass took a quarter of a million
// atomic additions (1024 workgroups x 256 bins), and the passes whose digit is spread over all
// bins ran at half the speed of the others.
constexpr int WIDE_HIST_THREADS = 1024;
constexpr int WIDE_HIST_GROUPS = 256;

__global__ __launch_bounds__(WIDE_HIST_THREADS) void wide_hist_kernel(const float* __restrict__ s, int n, int n_keep, int pass,
                                                                      uint32_t* __restrict__ ws, int share)
{
    // WIDE_COPIES counters per bin, side by side: lanes that hit the same bin (scores cluster in a
    // few exponents, so the first digit has a handful of busy bins) spread over as many addresses
    __shared__ uint32_t hist[256 * WIDE_COPIES];
    const int tid = threadIdx.x, lane = tid & 63;
    uint32_t prefix, mask, remaining;
    wide_replay(ws, pass, (uint32_t)n_keep, lane, prefix, mask, remaining);
    for (int q = tid; q < 256 * WIDE_COPIES; q += WIDE_HIST_THREADS) hist[q] = 0;
    __syncthreads();
    const int shift = 24 - 8 * pass;
    const int copy = lane & (WIDE_COPIES - 1);
    const int64_t lo64 = (int64_t)blockIdx.x * share;
    const int lo = (int)min<int64_t>(lo64, n), hi = (int)min<int64_t>(lo64 + share, n);
    for (int i0 = lo + tid; i0 < hi; i0 += 8 * WIDE_HIST_THREADS) {
        float v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = s[min(i0 + q * WIDE_HIST_THREADS, hi - 1)];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const uint32_t k = order_key(v[q]);
            if (i0 + q * WIDE_HIST_THREADS < hi && (k & mask) == prefix)
                atomicAdd(&hist[((k >> shift) & 255u) * WIDE_COPIES + copy], 1u);
        }
    }
    __syncthreads();
    if (tid < 256) {
        uint32_t mine = 0;
#pragma unroll
        for (int q = 0; q < WIDE_COPIES; ++q) mine += hist[tid * WIDE_COPIES + q];
        if (mine) atomicAdd(&ws[256 * pass + tid], mine);
    }
}

__global__ __launch_bounds__(WIDE_THREADS) void wide_count_kernel(const float* __restrict__ s, int n, int n_keep,
                                                                  uint32_t* __restrict__ ws)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t T, mask, need_eq;
    wide_replay(ws, 4, (uint32_t)n_keep, lane, T, mask, need_eq);
    if (blockIdx.x == 0 && tid == 0) { ws[WIDE_STATE] = T; ws[WIDE_STATE + 1] = need_eq; }
    const int group = blockIdx.x * (WIDE_THREADS / 64) + wave;
    const int lo = group * WIDE_WAVE_SLICE, hi = min(n, lo + WIDE_WAVE_SLICE);
    uint32_t gt = 0, eq = 0;
    for (int i0 = lo + lane; i0 < hi; i0 += 8 * 64) {
        float v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = s[min(i0 + q * 64, hi - 1)];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const uint32_t k = order_key(v[q]);
            if (i0 + q * 64 < hi) { gt += k > T; eq += k == T; }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) { gt += __shfl_down(gt, off, 64); eq += __shfl_down(eq, off, 64); }
    if (lane == 0 && lo < n) {
        ws[WIDE_COUNTS + group] = gt;
        ws[WIDE_COUNTS + WIDE_MAX_GROUPS + group] = eq;
    }
}

// exclusive prefix sums of the per-wavefront counts (groups <= 4096: four consecutive entries per thread)
__global__ __launch_bounds__(1024) void wide_scan_kernel(uint32_t* __restrict__ ws, int groups)
{
    __shared__ uint32_t wsum_gt[16], wsum_eq[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t g[4], e[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int j = 4 * tid + q;
        g[q] = j < groups ? ws[WIDE_COUNTS + j] : 0u;
        e[q] = j < groups ? ws[WIDE_COUNTS + WIDE_MAX_GROUPS + j] : 0u;
    }
    const uint32_t tg = g[0] + g[1] + g[2] + g[3], te = e[0] + e[1] + e[2] + e[3];
    uint32_t ig = tg, ie = te;                   // inclusive prefix inside the wavefront
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t a = __shfl_up(ig, off, 64), b = __shfl_up(ie, off, 64);
        if (lane >= off) { ig += a; ie += b; }
    }
    if (lane == 63) { wsum_gt[wave] = ig; wsum_eq[wave] = ie; }
    __syncthreads();
    uint32_t bg = ig - tg, be = ie - te;         // entries before this thread's four
    for (int w = 0; w < wave; ++w) { bg += wsum_gt[w]; be += wsum_eq[w]; }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int j = 4 * tid + q;
        if (j < groups) {
            ws[WIDE_COUNTS + 2 * WIDE_MAX_GROUPS + j] = bg;
            ws[WIDE_COUNTS + 3 * WIDE_MAX_GROUPS + j] = be;
        }
        bg += g[q];
        be += e[q];
    }
}

__global__ __launch_bounds__(WIDE_THREADS) void wide_write_kernel(const float* __restrict__ s, int n, int n_keep,
                                                                  const uint32_t* __restrict__ ws,
                                                                  int32_t* __restrict__ keep, int32_t* __restrict__ drop)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int group = blockIdx.x * (WIDE_THREADS / 64) + wave;
    const int lo = group * WIDE_WAVE_SLICE, hi = min(n, lo + WIDE_WAVE_SLICE);
    if (lo >= n) return;
    const uint32_t T = ws[WIDE_STATE], need_eq = ws[WIDE_STATE + 1];
    uint32_t run_gt = ws[WIDE_COUNTS + 2 * WIDE_MAX_GROUPS + group];
    uint32_t run_eq = ws[WIDE_COUNTS + 3 * WIDE_MAX_GROUPS + group];
    const uint64_t below = (1ull << lane) - 1ull;
    for (int base = lo; base < hi; base += 4 * 64) {
        float v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = s[min(base + q * 64 + lane, hi - 1)];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int i = base + q * 64 + lane;
            const uint32_t k = order_key(v[q]);
            const bool in = i < hi;
            const bool gt = in && k > T, eq = in && k == T;
            const uint64_t bgt = __ballot(gt);
            const uint64_t beq = __ballot(eq);
            const uint32_t pre_gt = run_gt + (uint32_t)__popcll(bgt & below);
            const uint32_t pre_eq = run_eq + (uint32_t)__popcll(beq & below);
            if (in) {
                const bool kept = gt || (eq && pre_eq < need_eq);
                const uint32_t kept_before = pre_gt + (pre_eq < need_eq ? pre_eq : need_eq);
                // (in range by construction; the comparisons make an out-of-range store impossible)
                if (kept) {
                    if (kept_before < (uint32_t)n_keep) keep[kept_before] = i;
                } else if (drop) {
                    const uint32_t pos = (uint32_t)i - kept_before;
                    if (pos < (uint32_t)(n - n_keep)) drop[pos] = i;
                }
            }
            run_gt += (uint32_t)__popcll(bgt);
            run_eq += (uint32_t)__popcll(beq);
        }
    }
}

__global__ void clear_flag_kernel(int32_t* flag) { *flag = 0; }

__global__ void validate_kernel(const int32_t* __restrict__ keep_idx, int n_keep, int n,
                                int32_t* __restrict__ flag)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_keep) return;
    const int v = keep_idx[i];
    bool bad = v < 0 || v >= n;
    if (i > 0 && keep_idx[i - 1] >= v) bad = true;
    if (bad) atomicOr(flag, 1);
}

}  // namespace

int launch_select(const float* scores, int n, int batch, int n_keep,
                  int32_t* keep_idx, int32_t* drop_idx, int64_t ld_idx, hipStream_t stream)
{
    const size_t key_bytes = (size_t)n * sizeof(uint32_t);
    if (n > SEL_LDS_KEYS)
        hipLaunchKernelGGL((select_kernel<false, SEL_THREADS>), dim3(batch), dim3(SEL_THREADS), 0, stream,
                           scores, n, n_keep, keep_idx, drop_idx, ld_idx);
    else if (batch >= 512)      // two workgroups per compute unit and more: throughput over latency
        hipLaunchKernelGGL((select_kernel<true, SEL_THREADS_MANY>), dim3(batch), dim3(SEL_THREADS_MANY), key_bytes,
                           stream, scores, n, n_keep, keep_idx, drop_idx, ld_idx);
    else
        hipLaunchKernelGGL((select_kernel<true, SEL_THREADS>), dim3(batch), dim3(SEL_THREADS), key_bytes, stream,
                           scores, n, n_keep, keep_idx, drop_idx, ld_idx);
    return hip_status(hipGetLastError());
}

size_t select_wide_workspace_bytes() { return WIDE_WORDS * sizeof(uint32_t); }

// shortest vector that goes to the many-workgroup path (below it the seven launches cost more
// than the single workgroup's passes)
int select_wide_min_n() { return 8 * WIDE_SLICE; }

int launch_select_wide(const float* scores, int n, int n_keep, int32_t* keep_idx, int32_t* drop_idx,
                       void* workspace, hipStream_t stream)
{
    uint32_t* ws = (uint32_t*)workspace;
    const int blocks = (n + WIDE_SLICE - 1) / WIDE_SLICE;
    const int groups = (n + WIDE_WAVE_SLICE - 1) / WIDE_WAVE_SLICE;        // wavefronts with scores
    if (groups > WIDE_MAX_GROUPS) return ZR_ERR_LIMIT;
    hipLaunchKernelGGL(wide_clear_kernel, dim3(1), dim3(1024), 0, stream, ws);
    const int hist_groups = std::min(WIDE_HIST_GROUPS, blocks);
    const int share = (n + hist_groups - 1) / hist_groups;
    for (int pass = 0; pass < 4; ++pass)
        hipLaunchKernelGGL(wide_hist_kernel, dim3(hist_groups), dim3(WIDE_HIST_THREADS), 0, stream, scores, n, n_keep, pass,
                           ws, share);
    hipLaunchKernelGGL(wide_count_kernel, dim3(blocks), dim3(WIDE_THREADS), 0, stream, scores, n, n_keep, ws);
    hipLaunchKernelGGL(wide_scan_kernel, dim3(1), dim3(1024), 0, stream, ws, groups);
    hipLaunchKernelGGL(wide_write_kernel, dim3(blocks), dim3(WIDE_THREADS), 0, stream, scores, n, n_keep,
                       (const uint32_t*)ws, keep_idx, drop_idx);
    return hip_status(hipGetLastError());
}

int launch_select_multi(const SelectMulti& m, int count, hipStream_t stream)
{
    int longest = 0;
    for (int b = 0; b < count; ++b) longest = std::max(longest, m.n[b]);
    const bool staged = longest <= SEL_LDS_KEYS;
    if (staged)
        hipLaunchKernelGGL(select_multi_kernel<true>, dim3(count), dim3(SEL_THREADS),
                           (size_t)longest * sizeof(uint32_t), stream, m);
    else
        hipLaunchKernelGGL(select_multi_kernel<false>, dim3(count), dim3(SEL_THREADS), 0, stream, m);
    return hip_status(hipGetLastError());
}

int launch_validate(const int32_t* keep_idx, int n_keep, int n, int32_t* flag, hipStream_t stream)
{
    // the flag is cleared by a kernel, not by a memset node
    hipLaunchKernelGGL(clear_flag_kernel, dim3(1), dim3(1), 0, stream, flag);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return ZR_ERR_HIP;
    const int threads = 256;
    hipLaunchKernelGGL(validate_kernel, dim3((n_keep + threads - 1) / threads), dim3(threads), 0,
                       stream, keep_idx, n_keep, n, flag);
    e = hipGetLastError();
    if (e != hipSuccess) return ZR_ERR_HIP;
    int32_t host = 0;
    e = hipMemcpyAsync(&host, flag, sizeof(int32_t), hipMemcpyDeviceToHost, stream);
    if (e != hipSuccess) return ZR_ERR_HIP;
    e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return ZR_ERR_HIP;
    return host ? ZR_ERR_INDEX : ZR_OK;
}

}  // namespace zr

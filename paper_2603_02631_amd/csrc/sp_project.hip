// sp_project: kept draft-token spans -> kept target tokens through character
// offsets (paper: Algorithm 1 "MapDraftChunksToTextSpans" and the target
// tokenisation of the kept text; Section 3.1).
//
// Target token t overlaps the character interval [cs, ce) of a draft span iff
//     target_off[t] < ce  and  target_off[t+1] > cs.
// With non-decreasing offsets the first condition holds on a prefix of t and
// the second on a suffix, so the overlapping tokens form the range
//     [ first t with target_off[t+1] > cs ,  first t with target_off[t] >= ce )
// found by two binary searches per span. Ranges of ascending spans are monotone,
// so ranges that overlap or touch are merged with an exclusive running maximum
// of the range ends and a prefix sum of "starts a new range" flags.
//
// Up to 1024 spans (the usual case: a few hundred kept chunks) take ONE launch,
// sp_project_one_kernel: workgroup 0 finds and merges the ranges, the other
// workgroups write the mask, each for itself and straight from the spans:
//   workgroup 0   stages a coarse index of the target offsets (every stride-th
//                 one, at most 4096) and the spans' character positions in LDS,
//                 narrows every search to one stride with a binary search of the
//                 index (one thread per search), finishes it with one wave-wide
//                 probe per search (several in flight per wave), and merges the
//                 ranges with the two scans described above;
//   mask groups   stage the spans' character intervals in LDS; since they are
//                 sorted, token [ts, te) is kept iff the first span that ends
//                 after ts begins before te: one LDS binary search per token.
// More spans take three launches:
//   sp_project_search_kernel one wave per (span, end): 64-ary search of the
//                            target offsets, three rounds of memory latency.
//   sp_project_spans_kernel  one workgroup: scans, merged target ranges,
//                            their count and the kept-token total.
//   sp_project_mask_kernel   one thread per target token: binary search of the
//                            merged ranges, writes the 0/1 keep mask.
#include "sp_common.hpp"

#include <algorithm>

namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / 64;

// 64-ary search by one wave: first index i in [0, n) with a[i] > v (STRICT) or a[i] >= v, n if
// none. Each round every lane probes one position; the predicate is monotone along the lanes, so
// a ballot gives the sub-interval. 64^3 > 2.6e5 positions take three rounds.
template <bool STRICT>
__device__ __forceinline__ int64_t wave_search(const int64_t *a, int64_t n, int64_t v, int lane)
{
    int64_t lo = 0, hi = n;                     // the answer lies in [lo, hi]
    while (lo < hi) {
        const int64_t cnt = hi - lo;
        const int64_t step = (cnt + 63) / 64;   // >= 1
        int64_t p = lo + (lane + 1) * step - 1;
        p = p < hi - 1 ? p : hi - 1;
        const int64_t val = a[p];
        const bool pass = STRICT ? (val > v) : (val >= v);
        const unsigned long long m = __ballot(pass);
        if (m == 0ull) { lo = hi; break; }      // the last lane probed hi - 1
        const int f = __ffsll((long long)m) - 1;
        int64_t pf = lo + (int64_t)(f + 1) * step - 1;
        pf = pf < hi - 1 ? pf : hi - 1;
        int64_t pprev = lo + (int64_t)f * step - 1;       // probe of lane f - 1 (fails); lo - 1 for f = 0
        pprev = pprev < hi - 1 ? pprev : hi - 1;
        hi = pf;
        lo = pprev + 1;
    }
    return lo;
}

struct ScanSmem {
    int64_t wave_max[kWavesPerBlock];
    int wave_sum[kWavesPerBlock];
};

// Inclusive block scans: running maximum of an int64 and running sum of an int.
__device__ __forceinline__ void block_scan(int64_t &mx, int &sum, ScanSmem &sm, int64_t &tot_max, int &tot_sum)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int64_t m2 = __shfl_up(mx, off);
        const int s2 = __shfl_up(sum, off);
        if (lane >= off) { mx = mx > m2 ? mx : m2; sum += s2; }
    }
    __syncthreads();
    if (lane == 63) { sm.wave_max[wave] = mx; sm.wave_sum[wave] = sum; }
    __syncthreads();
    int64_t bm = -1; int bs = 0;
    tot_max = -1; tot_sum = 0;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) {
        const int64_t wm = sm.wave_max[w];
        const int ws = sm.wave_sum[w];
        if (w < wave) { bm = bm > wm ? bm : wm; bs += ws; }
        tot_max = tot_max > wm ? tot_max : wm;
        tot_sum += ws;
    }
    mx = mx > bm ? mx : bm;
    sum += bs;
}

// Raw target range of every span: tspans[2s] = first t with target_off[t+1] > cs,
// tspans[2s+1] = first t with target_off[t] >= ce (M if none).
__global__ __launch_bounds__(kThreads) void sp_project_search_kernel(
    const int64_t *__restrict__ draft_off, int64_t L, const int64_t *__restrict__ target_off, int64_t M,
    const int64_t *__restrict__ spans, const int32_t *__restrict__ n_spans_p, int max_spans, int64_t *tspans)
{
    const int lane = threadIdx.x & 63;
    const int gw = blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    const int s = gw >> 1, end = gw & 1;
    int n_spans = *n_spans_p;
    if (n_spans > max_spans) n_spans = max_spans;
    if (s >= n_spans) return;
    int64_t tok = spans[2 * s + end];
    tok = tok < 0 ? 0 : (tok > L ? L : tok);
    const int64_t ch = draft_off[tok];
    const int64_t r = end == 0 ? wave_search<true>(target_off + 1, M, ch, lane) : wave_search<false>(target_off, M, ch, lane);
    if (lane == 0) tspans[2 * s + end] = r;
}

__global__ __launch_bounds__(kThreads) void sp_project_spans_kernel(
    const int32_t *__restrict__ n_spans_p, int max_spans, int64_t *tspans, int32_t *n_tspans, int64_t *n_kept)
{
    __shared__ ScanSmem sm;
    __shared__ int64_t red[kWavesPerBlock];
    const int tid = threadIdx.x;
    int n_spans = *n_spans_p;
    if (n_spans > max_spans) n_spans = max_spans;
    if (n_spans < 0) n_spans = 0;

    int64_t carry_hi = -1;      // largest range end seen in earlier segments (-1: none)
    int carry_n = 0;            // merged ranges opened in earlier segments
    for (int base = 0; base < n_spans; base += kThreads) {
        const int s = base + tid;
        int64_t lo = 0, hi = 0;
        bool nonempty = false;
        if (s < n_spans) {          // raw range from the search kernel; merged ranges are written back in place
            lo = tspans[2 * s];     // (an entry is overwritten only after its segment has been read: r <= s)
            hi = tspans[2 * s + 1];
            nonempty = lo < hi;
        }
        // exclusive running maximum of the ends of earlier non-empty ranges
        int64_t incl_max = nonempty ? hi : -1;
        int dummy = 0;
        int64_t tot_max; int tot_dummy;
        block_scan(incl_max, dummy, sm, tot_max, tot_dummy);
        int64_t prev_hi = __shfl_up(incl_max, 1);
        if ((tid & 63) == 0) {
            prev_hi = -1;
            for (int w = 0; w < (tid >> 6); ++w) prev_hi = prev_hi > sm.wave_max[w] ? prev_hi : sm.wave_max[w];
        }
        prev_hi = prev_hi > carry_hi ? prev_hi : carry_hi;
        const int start = nonempty && (prev_hi < 0 || lo > prev_hi);
        int id = start;
        int64_t dm = -1; int64_t tm; int tot_start;
        block_scan(dm, id, sm, tm, tot_start);
        if (start) {
            const int r = carry_n + id - 1;
            tspans[2 * r] = lo;
            if (r > 0) tspans[2 * (r - 1) + 1] = prev_hi;   // closes the previous merged range
        }
        carry_hi = carry_hi > tot_max ? carry_hi : tot_max;
        carry_n += tot_start;
    }
    if (tid == 0) {
        if (carry_n > 0) tspans[2 * (carry_n - 1) + 1] = carry_hi;
        *n_tspans = carry_n;
    }
    __syncthreads();
    // kept-token total = sum of merged range lengths
    int64_t part = 0;
    for (int r = tid; r < carry_n; r += kThreads) part += tspans[2 * r + 1] - tspans[2 * r];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) part += __shfl_xor(part, off);
    if ((tid & 63) == 0) red[tid >> 6] = part;
    __syncthreads();
    if (tid == 0) {
        int64_t t = 0;
        for (int w = 0; w < kWavesPerBlock; ++w) t += red[w];
        *n_kept = t;
    }
}

__global__ __launch_bounds__(kThreads) void sp_project_mask_kernel(const int64_t *__restrict__ tspans,
                                                                   const int32_t *__restrict__ n_tspans, int64_t M,
                                                                   uint8_t *__restrict__ mask)
{
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (t >= M) return;
    const int n = *n_tspans;
    // last merged range whose begin is <= t
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = lo + ((hi - lo) >> 1);
        if (tspans[2 * mid] <= t) lo = mid + 1; else hi = mid;
    }
    uint8_t keep = 0;
    if (lo > 0 && t < tspans[2 * (lo - 1) + 1]) keep = 1;
    mask[t] = keep;
}

// ---------------------------------------------------------------------------
// one launch for up to kOneSpans spans
// ---------------------------------------------------------------------------
constexpr int kOneThreads = 1024;
constexpr int kOneWaves = kOneThreads / 64;
constexpr int kOneSpans = 1024;              // spans the single launch holds in LDS
static_assert(kOneSpans == kOneThreads, "the merge scan takes one span per thread");
constexpr int kCoarse = 4096;                // entries of the coarse index
constexpr int kMaskPerThread = 2;            // target tokens per thread of a mask workgroup: one prompt (more, smaller workgroups) ...
constexpr int kMaskPerThreadBatch = 8;       // ... a ragged batch (measured: 14.8 vs 17.5 µs and 19.6 vs 30.4 µs)

struct OneSmem {
    int64_t coarse[kCoarse];                 // target_off[i * stride]
    int64_t ch[2 * kOneSpans];               // character position of (span, end)
    int32_t win[2 * kOneSpans];              // first position of each search's window
    int32_t range[2 * kOneSpans];            // raw target range of every span
    int32_t wave_max[kOneWaves];
    int32_t wave_sum[kOneWaves];
    int64_t red[kOneWaves];
};

// Inclusive block scans over kOneThreads threads: running maximum and running sum (token positions
// fit 32 bits on this path).
__device__ __forceinline__ void block_scan_one(int &mx, int &sum, OneSmem &sm, int &tot_max, int &tot_sum)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int m2 = __shfl_up(mx, off);
        const int s2 = __shfl_up(sum, off);
        if (lane >= off) { mx = mx > m2 ? mx : m2; sum += s2; }
    }
    __syncthreads();
    if (lane == 63) { sm.wave_max[wave] = mx; sm.wave_sum[wave] = sum; }
    __syncthreads();
    int bm = -1, bs = 0;
    tot_max = -1; tot_sum = 0;
#pragma unroll
    for (int w = 0; w < kOneWaves; ++w) {
        const int wm = sm.wave_max[w];
        const int ws = sm.wave_sum[w];
        if (w < wave) { bm = bm > wm ? bm : wm; bs += ws; }
        tot_max = tot_max > wm ? tot_max : wm;
        tot_sum += ws;
    }
    mx = mx > bm ? mx : bm;
    sum += bs;
}

__device__ __forceinline__ int64_t read_lane64(int64_t v, int l)
{
    const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)(uint64_t)v, l);
    const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)v >> 32), l);
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// Requires max_spans <= kOneSpans (one scan segment: kOneSpans == kOneThreads) and M < 2^31.
template <int kMaskPerThread>
__device__ __forceinline__ void project_one_body(
    const int64_t *__restrict__ draft_off, int64_t L, const int64_t *__restrict__ target_off, int M,
    const int64_t *__restrict__ spans, const int32_t *__restrict__ n_spans_p, int max_spans, int stride,
    int n_coarse, int64_t *__restrict__ tspans, int32_t *__restrict__ n_tspans, int64_t *__restrict__ n_kept,
    uint8_t *__restrict__ mask)
{
    __shared__ OneSmem sm;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // character position of every (span, end): ch[2s] = begin, ch[2s + 1] = end of span s. All max_spans
    // entries of the buffer are read, so that this does not wait for the count; those past it are not used.
    for (int i = tid; i < 2 * max_spans; i += kOneThreads) {
        int64_t tok = spans[i];
        tok = tok < 0 ? 0 : (tok > L ? L : tok);
        sm.ch[i] = draft_off[tok];
    }
    int n_spans = *n_spans_p;
    if (n_spans > max_spans) n_spans = max_spans;
    if (n_spans < 0) n_spans = 0;

    if (blockIdx.x > 0) {
        // ---- mask workgroup ----
        __syncthreads();
        const int base = ((int)blockIdx.x - 1) * (kOneThreads * kMaskPerThread);
#pragma unroll
        for (int k = 0; k < kMaskPerThread; ++k) {
            const int t = base + k * kOneThreads + tid;
            if (t >= M) break;
            const int64_t ts = target_off[t], te = target_off[t + 1];
            int lo = 0, hi = n_spans;          // first span whose end lies after ts
            while (lo < hi) {
                const int mid = lo + ((hi - lo) >> 1);
                if (sm.ch[2 * mid + 1] > ts) hi = mid; else lo = mid + 1;
            }
            mask[t] = (lo < n_spans && sm.ch[2 * lo] < te) ? 1 : 0;
        }
        return;
    }

    // ---- workgroup 0: ranges ----
    for (int i = tid; i < n_coarse; i += kOneThreads) {
        const int p = i * stride;
        sm.coarse[i] = target_off[p < M ? p : M];
    }
    __syncthreads();
    // Search q = (span, end) looks for the first position p of target_off that passes its test:
    // end 0: target_off[p] > ch over p in [1, M], result p - 1; end 1: target_off[p] >= ch over
    // p in [0, M), result p; M when nothing passes. The index narrows it to one stride.
    const int n_q = 2 * n_spans;
    for (int q = tid; q < n_q; q += kOneThreads) {
        const int64_t ch = sm.ch[q];
        const bool strict = (q & 1) == 0;
        int lo = 0, hi = n_coarse;             // first index entry that passes
        while (lo < hi) {
            const int mid = lo + ((hi - lo) >> 1);
            const int64_t v = sm.coarse[mid];
            if (strict ? (v > ch) : (v >= ch)) hi = mid; else lo = mid + 1;
        }
        // entries below lo fail, entry lo (if any) passes: the answer is in ((lo - 1) * stride, lo * stride]
        sm.win[q] = lo > 0 ? (lo - 1) * stride + 1 : 0;
    }
    __syncthreads();
    // One wave-wide probe per search finishes it (stride <= 63). Searches go to the waves in groups
    // of kGroup, dealt round robin; a wave has kPass groups in flight. What is the same for all lanes of
    // a search stays in scalar registers, and lane l < kGroup * kPass finishes search l of the pass.
    // A window needs no bounds: lanes past position M read position M again, which cannot come before
    // the first passing position, and position 0 passing a search over [1, M] gives the same result 0.
    constexpr int kGroup = 8, kPass = 4;
    for (int g0 = wave; g0 * kGroup < n_q; g0 += kOneWaves * kPass) {
        const int ql = (g0 + (lane >> 3) * kOneWaves) * kGroup + (lane & 7);
        const bool has = lane < kGroup * kPass && ql < n_q;
        int first_v = 0;
        int64_t ch_v = 0;
        if (has) { first_v = sm.win[ql]; ch_v = sm.ch[ql]; }
        int64_t val[kGroup * kPass];
#pragma unroll
        for (int g = 0; g < kPass; ++g) {
            if ((g0 + g * kOneWaves) * kGroup >= n_q) break;                  // uniform
#pragma unroll
            for (int u = 0; u < kGroup; ++u) {
                const int first = __builtin_amdgcn_readlane(first_v, g * kGroup + u);
                const int room = M - first;
                val[g * kGroup + u] = target_off[first + (lane < room ? lane : room)];
            }
        }
        uint32_t m_lo = 0, m_hi = 0;             // lane l: which lanes pass search l
#pragma unroll
        for (int g = 0; g < kPass; ++g) {
            if ((g0 + g * kOneWaves) * kGroup >= n_q) break;
#pragma unroll
            for (int u = 0; u < kGroup; ++u) {
                const int l = g * kGroup + u;
                const int64_t ch = read_lane64(ch_v, l);
                const bool pass = (u & 1) == 0 ? (val[l] > ch) : (val[l] >= ch);     // ql is even for even u
                const unsigned long long m = __ballot(pass);
                m_lo = lane == l ? (uint32_t)m : m_lo;
                m_hi = lane == l ? (uint32_t)(m >> 32) : m_hi;
            }
        }
        if (has) {
            const unsigned long long m = ((unsigned long long)m_hi << 32) | m_lo;
            // nothing passes within the window: only in the last window, i.e. nothing passes at all
            int res = M;
            if (m != 0ull) {
                res = first_v + (__ffsll((long long)m) - 1) - ((lane & 1) == 0 ? 1 : 0);
                res = res > 0 ? res : 0;
            }
            sm.range[ql] = res;
        }
    }
    __syncthreads();

    // merge overlapping / touching ranges (see the file header): one segment, thread s has span s
    int lo = 0, hi = 0;
    bool nonempty = false;
    if (tid < n_spans) {
        lo = sm.range[2 * tid];
        hi = sm.range[2 * tid + 1];
        nonempty = lo < hi;
    }
    int incl_max = nonempty ? hi : -1;
    int dummy = 0, tot_max, tot_dummy;
    block_scan_one(incl_max, dummy, sm, tot_max, tot_dummy);
    int prev_hi = __shfl_up(incl_max, 1);      // exclusive running maximum of the ends of earlier ranges
    if (lane == 0) {
        prev_hi = -1;
        for (int w = 0; w < wave; ++w) prev_hi = prev_hi > sm.wave_max[w] ? prev_hi : sm.wave_max[w];
    }
    const int start = nonempty && (prev_hi < 0 || lo > prev_hi);
    int id = start, dm = -1, tm, n_merged;
    block_scan_one(dm, id, sm, tm, n_merged);
    if (start) {
        const int r = id - 1;
        tspans[2 * r] = lo;
        if (r > 0) tspans[2 * (r - 1) + 1] = prev_hi;      // closes the previous merged range
    }
    if (tid == 0) {
        if (n_merged > 0) tspans[2 * (n_merged - 1) + 1] = tot_max;
        *n_tspans = n_merged;
    }
    // kept tokens: each range adds its part beyond every earlier end
    int64_t part = 0;
    if (nonempty) {
        const int from = lo > prev_hi ? lo : prev_hi;
        part = hi > from ? hi - from : 0;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) part += __shfl_xor(part, off);
    if (lane == 0) sm.red[wave] = part;
    __syncthreads();
    if (tid == 0) {
        int64_t t = 0;
        for (int w = 0; w < kOneWaves; ++w) t += sm.red[w];
        *n_kept = t;
    }
}

__global__ __launch_bounds__(kOneThreads) void sp_project_one_kernel(
    const int64_t *__restrict__ draft_off, int64_t L, const int64_t *__restrict__ target_off, int M,
    const int64_t *__restrict__ spans, const int32_t *__restrict__ n_spans_p, int max_spans, int stride,
    int n_coarse, int64_t *__restrict__ tspans, int32_t *__restrict__ n_tspans, int64_t *__restrict__ n_kept,
    uint8_t *__restrict__ mask)
{
    project_one_body<kMaskPerThread>(draft_off, L, target_off, M, spans, n_spans_p, max_spans, stride, n_coarse, tspans,
                                     n_tspans, n_kept, mask);
}

// Ragged batch: prompt b = blockIdx.y. Its L_b + 1 draft offsets start at off[b] + b of the packed array,
// its M_b + 1 target offsets at moff[b] + b, its spans and target ranges (k_b of each at most) at
// kept_off[b], its mask bytes at moff[b]. Workgroup 0 of a prompt finds its ranges, the others its mask.
__global__ __launch_bounds__(kOneThreads) void sp_project_batch_kernel(
    const int64_t *__restrict__ draft_off, const int64_t *__restrict__ off, const int64_t *__restrict__ target_off,
    const int64_t *__restrict__ moff, const int64_t *__restrict__ spans, const int32_t *__restrict__ n_spans,
    const int64_t *__restrict__ kept_off, int64_t *__restrict__ tspans, int32_t *__restrict__ n_tspans,
    int64_t *__restrict__ n_kept, uint8_t *__restrict__ mask)
{
    const int b = blockIdx.y;
    const int64_t o = off[b], L = off[b + 1] - o, mo = moff[b];
    const int M = (int)(moff[b + 1] - mo);
    const int64_t k0 = kept_off[b];
    const int max_spans = (int)(kept_off[b + 1] - k0);
    if (blockIdx.x > 0 && ((int64_t)blockIdx.x - 1) * (kOneThreads * kMaskPerThreadBatch) >= M) return;   // past this prompt's mask
    if (L < 1 || M < 1 || max_spans < 1) {           // nothing kept (uniform: no barrier is skipped by part of a workgroup)
        if (blockIdx.x == 0 && threadIdx.x == 0) { n_tspans[b] = 0; n_kept[b] = 0; }
        if (blockIdx.x > 0 && mask)
            for (int k = 0; k < kMaskPerThreadBatch; ++k) {
                const int64_t t = ((int64_t)blockIdx.x - 1) * (kOneThreads * kMaskPerThreadBatch) + (int64_t)k * kOneThreads + threadIdx.x;
                if (t < M) mask[mo + t] = 0;
            }
        return;
    }
    if (blockIdx.x > 0 && !mask) return;
    const int stride = (M + kCoarse) / kCoarse;          // ceil((M + 1) / kCoarse)
    const int n_coarse = (M + stride) / stride;          // ceil((M + 1) / stride)
    project_one_body<kMaskPerThreadBatch>(draft_off + o + b, L, target_off + mo + b, M, spans + 2 * k0, n_spans + b, max_spans, stride,
                     n_coarse, tspans + 2 * k0, n_tspans + b, n_kept + b, mask ? mask + mo : nullptr);
}

}  // namespace

extern "C" sp_status sp_project(const int64_t *draft_off_dev, int64_t L, const int64_t *target_off_dev, int64_t M,
                                const int64_t *spans_dev, const int32_t *n_spans_dev, int32_t max_spans,
                                int64_t *tspans_dev, int32_t *n_tspans_dev, uint8_t *keep_mask_dev,
                                int64_t *n_kept_dev, void *hip_stream)
{
    if (!draft_off_dev || !target_off_dev || !spans_dev || !n_spans_dev || !tspans_dev || !n_tspans_dev || !n_kept_dev)
        return sp::fail(SP_ERR_INVALID_ARG, "only keep_mask_dev may be null");
    if (L < 1 || M < 1) return sp::fail(SP_ERR_INVALID_ARG, "L = %lld and M = %lld must be >= 1", (long long)L, (long long)M);
    if (max_spans < 1 || max_spans > (1 << 24))
        return sp::fail(SP_ERR_INVALID_ARG, "max_spans = %d outside 1..2^24", max_spans);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    // one launch when the spans fit its LDS and one stride of the coarse index fits a wave-wide probe
    const int64_t stride = M / kCoarse + 1;          // ceil((M + 1) / kCoarse)
    if (max_spans <= kOneSpans && stride <= 63) {
        const int n_coarse = (int)sp::ceil_div(M + 1, stride);
        const int64_t mask_groups = keep_mask_dev ? sp::ceil_div(M, (int64_t)kOneThreads * kMaskPerThread) : 0;
        hipLaunchKernelGGL(sp_project_one_kernel, dim3((unsigned)(1 + mask_groups)), dim3(kOneThreads), 0, st, draft_off_dev, L,
                           target_off_dev, (int)M, spans_dev, n_spans_dev, (int)max_spans, (int)stride, n_coarse, tspans_dev,
                           n_tspans_dev, n_kept_dev, keep_mask_dev);
        SP_HIP_CHECK(hipGetLastError());
        return SP_OK;
    }
    const unsigned search_grid = (unsigned)((2 * (int64_t)max_spans + kWavesPerBlock - 1) / kWavesPerBlock);
    hipLaunchKernelGGL(sp_project_search_kernel, dim3(search_grid), dim3(kThreads), 0, st, draft_off_dev, L,
                       target_off_dev, M, spans_dev, n_spans_dev, (int)max_spans, tspans_dev);
    SP_HIP_CHECK(hipGetLastError());
    hipLaunchKernelGGL(sp_project_spans_kernel, dim3(1), dim3(kThreads), 0, st, n_spans_dev, (int)max_spans,
                       tspans_dev, n_tspans_dev, n_kept_dev);
    SP_HIP_CHECK(hipGetLastError());
    if (keep_mask_dev) {
        const unsigned grid = (unsigned)((M + kThreads - 1) / kThreads);
        hipLaunchKernelGGL(sp_project_mask_kernel, dim3(grid), dim3(kThreads), 0, st, (const int64_t *)tspans_dev,
                           (const int32_t *)n_tspans_dev, M, keep_mask_dev);
        SP_HIP_CHECK(hipGetLastError());
    }
    return SP_OK;
}

extern "C" sp_status sp_project_batch(const int64_t *draft_off_dev, const int64_t *offsets_host,
                                      const int64_t *offsets_dev, const int64_t *target_off_dev,
                                      const int64_t *moffsets_host, const int64_t *moffsets_dev, int32_t B,
                                      const int64_t *spans_dev, const int32_t *n_spans_dev,
                                      const int64_t *kept_off_host, const int64_t *kept_off_dev, int64_t *tspans_dev,
                                      int32_t *n_tspans_dev, uint8_t *keep_mask_dev, int64_t *n_kept_dev,
                                      void *hip_stream)
{
    if (!draft_off_dev || !offsets_host || !offsets_dev || !target_off_dev || !moffsets_host || !moffsets_dev ||
        !spans_dev || !n_spans_dev || !kept_off_host || !kept_off_dev || !tspans_dev || !n_tspans_dev || !n_kept_dev)
        return sp::fail(SP_ERR_INVALID_ARG, "only keep_mask_dev may be null");
    if (B < 1 || B > 4096) return sp::fail(SP_ERR_INVALID_ARG, "B = %d (supported: 1..4096)", B);
    if (offsets_host[0] != 0 || moffsets_host[0] != 0 || kept_off_host[0] != 0)
        return sp::fail(SP_ERR_INVALID_ARG, "offsets_host[0], moffsets_host[0] and kept_off_host[0] must be 0");
    int64_t max_m = 0;
    for (int b = 0; b < B; ++b) {
        const int64_t len = offsets_host[b + 1] - offsets_host[b], m = moffsets_host[b + 1] - moffsets_host[b],
                      k = kept_off_host[b + 1] - kept_off_host[b];
        if (len < 0 || m < 0 || k < 0) return sp::fail(SP_ERR_INVALID_ARG, "offsets decrease at prompt %d", b);
        if (k > kOneSpans)
            return sp::fail(SP_ERR_UNSUPPORTED, "prompt %d: %lld spans (the batch call supports <= %d a prompt; use sp_project)",
                            b, (long long)k, kOneSpans);
        if (m >= (int64_t)63 * kCoarse)
            return sp::fail(SP_ERR_UNSUPPORTED, "prompt %d: %lld target tokens (the batch call supports < %d a prompt; use sp_project)",
                            b, (long long)m, 63 * kCoarse);
        max_m = std::max(max_m, m);
    }
    const int64_t mask_groups = keep_mask_dev ? sp::ceil_div(max_m, (int64_t)kOneThreads * kMaskPerThreadBatch) : 0;
    hipLaunchKernelGGL(sp_project_batch_kernel, dim3((unsigned)(1 + mask_groups), (unsigned)B), dim3(kOneThreads), 0,
                       static_cast<hipStream_t>(hip_stream), draft_off_dev, offsets_dev, target_off_dev, moffsets_dev,
                       spans_dev, n_spans_dev, kept_off_dev, tspans_dev, n_tspans_dev, n_kept_dev, keep_mask_dev);
    SP_HIP_CHECK(hipGetLastError());
    return SP_OK;
}

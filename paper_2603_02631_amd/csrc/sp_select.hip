// sp_select: average pooling, chunk means, top-k chunks, merged spans
// (paper: Algorithm 1 "AvgPool1D", "PartitionIntoChunks", "TopKChunks",
// "MergeAdjacentChunks"; Appendix A.1.2; Appendix A.3).
//
// Two kernels:
//   sp_chunk_kernel  one wavefront per chunk. The wave stages the chunk's
//                    scores plus a (w-1)/2 halo through its own LDS slice in
//                    segments, each lane forms the window sums of four
//                    consecutive tokens, and a fixed-order shuffle tree gives
//                    the chunk mean. The pooled vector is never written out.
//   sp_topk_kernel   one workgroup. MSB-first radix select (4 passes of 8 bits)
//                    on order-preserving integer images of the fp32 chunk
//                    scores finds the k-th largest score exactly; chunks above
//                    it are kept, chunks equal to it are kept in index order
//                    until k is reached (lower index wins a tie). Two block
//                    scans then emit the kept indices in ascending order and
//                    the merged spans.
// Everything is integer or fixed-order fp32 work, so results are deterministic.
//
// sp_select_budget (Section 3.1: a fixed target-side length of the compressed
// prompt) finds k on the device instead of taking it from the host. With
// rank[j] = position of chunk j in the order (score descending, index
// ascending), the top-k chunks are those of rank < k, and whether target token t
// is kept by the top-k chunks depends on k only through one number r(t): a token
// with at least one character is kept iff some chunk whose character interval it
// overlaps is selected, r(t) = the smallest rank among those chunks; a token
// without characters is kept iff it lies strictly inside a merged span, i.e.
// inside one chunk or on a boundary whose chunks on both sides are all selected,
// r(t) = the largest rank among them. Kept tokens at k = #{t : r(t) < k}: a
// histogram of r and a prefix sum give the count for every k at once.
//   sp_chunk_kernel       also leaves the chunk boundaries' character offsets in a
//                         compact array and clears the counters of the next two;
//   sp_rank_kernel        rank of every chunk by counting: tiles of 256 chunks
//                         against tiles of 256 chunks, one workgroup per pair;
//   sp_token_rank_kernel  one thread per target token: binary searches of the
//                         compact boundary array, r(t), histogram;
//   sp_budget_kernel      one workgroup: prefix sum, largest k within the budget;
//   sp_topk_kernel        as above, reading k from device memory.
#include "sp_common.hpp"

#include <algorithm>
#include <atomic>

namespace {

constexpr int kChunkThreads = 256;           // 4 waves, one chunk each
constexpr int kSeg = 256;                    // tokens staged per wave per step
constexpr int kMaxPool = 129;                // halo (w-1)/2 <= 64 fits the staging slice
constexpr int kSegLds = kSeg + kMaxPool - 1; // staged floats per wave
constexpr int kTopkThreads = 1024;

__device__ __forceinline__ void chunk_body(const float *__restrict__ scores, int64_t L, int pool_w, int chunk,
                                           int64_t n_chunks, float *__restrict__ cs_ws, float *__restrict__ cs_out,
                                           const int64_t *__restrict__ draft_off, int64_t *__restrict__ bnd,
                                           int32_t *__restrict__ rank, int32_t *__restrict__ hist)
{
    __shared__ float stage[kChunkThreads / 64][kSegLds + 3];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t ci = (int64_t)blockIdx.x * (kChunkThreads / 64) + wave;
    if (ci >= n_chunks) return;              // whole wave leaves together; no block barrier is used
    float *st = stage[wave];
    const int half = (pool_w - 1) / 2;
    const int64_t begin = ci * chunk;
    const int64_t end = (begin + chunk < L) ? begin + chunk : L;
    float part = 0.f;
    for (int64_t seg = begin; seg < end; seg += kSeg) {
        const int n_tok = (int)((end - seg < kSeg) ? end - seg : kSeg);
        const int n_stage = n_tok + 2 * half;
        for (int i = lane; i < n_stage; i += 64) {
            const int64_t j = seg - half + i;
            st[i] = (j >= 0 && j < L) ? scores[j] : 0.f;
        }
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        // lane handles tokens 4*lane .. 4*lane+3 of the segment; each window is summed on its own
        const int t0 = 4 * lane;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (t0 + e < n_tok) {
                float win = 0.f;
                for (int i = 0; i < pool_w; ++i) win += st[t0 + e + i];
                part += win;
            }
        }
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) part += __shfl_xor(part, off);
    if (lane == 0) {
        const float v = part / ((float)pool_w * (float)(end - begin)) + 0.0f;
        cs_ws[ci] = v;
        if (cs_out) cs_out[ci] = v;
        if (bnd) {
            // set-up for the budget search: character offset of the chunk's first token (one more entry:
            // the end of the text), cleared rank counters and histogram bins (one more: "never kept")
            bnd[ci] = draft_off[begin];
            rank[ci] = 0;
            hist[ci] = 0;
            if (ci == n_chunks - 1) {
                bnd[n_chunks] = draft_off[L];
                hist[n_chunks] = 0;
            }
        }
    }
}

__global__ __launch_bounds__(kChunkThreads) void sp_chunk_kernel(const float *__restrict__ scores, int64_t L,
                                                                 int pool_w, int chunk, int64_t n_chunks,
                                                                 float *__restrict__ cs_ws,
                                                                 float *__restrict__ cs_out,
                                                                 const int64_t *__restrict__ draft_off,
                                                                 int64_t *__restrict__ bnd,
                                                                 int32_t *__restrict__ rank,
                                                                 int32_t *__restrict__ hist)
{
    chunk_body(scores, L, pool_w, chunk, n_chunks, cs_ws, cs_out, draft_off, bnd, rank, hist);
}

// Ragged batch: prompt b = blockIdx.y owns scores [off[b], off[b+1]) and the chunk-score slots from
// off[b] / chunk + b on (distinct prompts' slots cannot overlap: a prompt has at most
// off[b+1] / chunk - off[b] / chunk + 1 chunks).
__device__ __forceinline__ int64_t batch_chunk_slot(int64_t off_b, int b, int chunk) { return off_b / chunk + b; }

__global__ __launch_bounds__(kChunkThreads) void sp_chunk_batch_kernel(const float *__restrict__ scores,
                                                                       const int64_t *__restrict__ off, int pool_w,
                                                                       int chunk, float *__restrict__ cs_ws,
                                                                       float *__restrict__ cs_out)
{
    const int b = blockIdx.y;
    const int64_t o = off[b], L = off[b + 1] - o;
    const int64_t n_chunks = (L + chunk - 1) / chunk;
    if ((int64_t)blockIdx.x * (kChunkThreads / 64) >= n_chunks) return;        // also: empty prompt
    const int64_t slot = batch_chunk_slot(o, b, chunk);
    chunk_body(scores + o, L, pool_w, chunk, n_chunks, cs_ws + slot, cs_out ? cs_out + slot : nullptr, nullptr, nullptr,
               nullptr, nullptr);
}

// fp32 -> uint32 whose unsigned order is the float order (-0 mapped onto +0 first).
__device__ __forceinline__ uint32_t order_key(float v)
{
    const uint32_t u = __float_as_uint(v + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Inclusive block scan of one int per thread (1024 threads = 16 waves).
__device__ __forceinline__ int block_scan_incl(int v, int *wave_tot /*[16]*/, int &block_total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int x = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int y = __shfl_up(x, off);
        if (lane >= off) x += y;
    }
    __syncthreads();                         // protects wave_tot from the previous use
    if (lane == 63) wave_tot[wave] = x;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kTopkThreads / 64; ++w) {
        const int t = wave_tot[w];
        if (w < wave) base += t;
        tot += t;
    }
    block_total = tot;
    return x + base;
}

// R > 0: the keys of up to R * 1024 chunks are read once and kept in registers (every pass over the
// chunk scores would otherwise pay a trip to memory); R = 0: any number of chunks, re-read per pass.
template <int R>
__device__ __forceinline__ void topk_body(const float *__restrict__ cs, int64_t n_chunks, int64_t k,
                                          const int64_t *__restrict__ k_dev, int chunk, int64_t L, int32_t *sel,
                                          int64_t *__restrict__ spans, int32_t *__restrict__ n_spans)
{
    __shared__ int hist[256];
    if (k_dev) {                             // k chosen on the device (budget search); always within 1..n_chunks
        k = *k_dev;
        k = k < 1 ? 1 : (k > n_chunks ? n_chunks : k);
    }
    __shared__ int wave_tot[kTopkThreads / 64];
    __shared__ uint32_t s_prefix;
    __shared__ int64_t s_need;
    const int tid = threadIdx.x;

    uint32_t cached[R > 0 ? R : 1];
    if (R > 0) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int64_t i = (int64_t)r * kTopkThreads + tid;
            cached[r] = i < n_chunks ? order_key(cs[i]) : 0u;
        }
    }
    // key of chunk i = seg * kTopkThreads + tid (seg is a compile-time index wherever R > 0)
    auto key_of = [&](int seg, int64_t i) -> uint32_t { return R > 0 ? cached[seg] : order_key(cs[i]); };

    // ---- radix select: key of the k-th largest chunk score ----
    // Per pass: all threads count their candidates into a 256-bin histogram; wave 0 alone scans the
    // bins from the top (four per lane, one shuffle scan), picks the bin that holds the k-th, and clears
    // the histogram for the next pass: two barriers per pass.
    uint32_t prefix = 0, mask = 0;
    int64_t need = k;                        // how many still to take from the current bucket
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (R > 0) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int64_t i = (int64_t)r * kTopkThreads + tid;
                const uint32_t key = cached[r];
                if (i < n_chunks && (key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
            }
        } else {
            for (int64_t i = tid; i < n_chunks; i += kTopkThreads) {
                const uint32_t key = order_key(cs[i]);
                if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
            }
        }
        __syncthreads();
        if (tid < 64) {
            // lane l owns bins 255-4l .. 252-4l, in that (descending) order
            int h[4], lane_sum = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                h[j] = hist[255 - 4 * tid - j];
                hist[255 - 4 * tid - j] = 0;
                lane_sum += h[j];
            }
            int incl = lane_sum;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int y = __shfl_up(incl, off);
                if (tid >= off) incl += y;
            }
            int64_t before = incl - lane_sum;        // candidates in the bins above this lane's
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (before < need && before + h[j] >= need) {
                    s_prefix = prefix | ((uint32_t)(255 - 4 * tid - j) << shift);
                    s_need = need - before;
                }
                before += h[j];
            }
        }
        __syncthreads();
        prefix = s_prefix;
        need = s_need;
        mask |= 255u << shift;
    }
    const uint32_t thr = prefix;             // exact key of the k-th largest score
    // `need` = number of chunks equal to thr to keep, taken in index order.

    // ---- emit kept chunk indices in ascending order ----
    // Kept: every chunk above thr and the first `need` chunks equal to thr. One scan per segment of a
    // packed pair (above in the low half, equal in the high half) gives each chunk's output position:
    // chunks above before it plus min(equal chunks before it, need).
    int64_t eq_seen = 0, gt_seen = 0;
    const int n_seg = (int)((n_chunks + kTopkThreads - 1) / kTopkThreads);
#pragma unroll
    for (int seg = 0; seg < (R > 0 ? R : n_seg); ++seg) {
        if (R > 0 && seg >= n_seg) break;            // uniform
        const int64_t base = (int64_t)seg * kTopkThreads;
        const int64_t i = base + tid;
        uint32_t key = 0;
        if (i < n_chunks) key = key_of(seg, i);
        const int is_eq = (i < n_chunks && key == thr) ? 1 : 0;
        const int is_gt = (i < n_chunks && key > thr) ? 1 : 0;
        int total;
        const int incl = block_scan_incl(is_gt | (is_eq << 16), wave_tot, total);
        const int64_t gt_before = gt_seen + (incl & 0xffff) - is_gt;
        const int64_t eq_before = eq_seen + (incl >> 16) - is_eq;
        if (is_gt) sel[gt_before + (eq_before < need ? eq_before : need)] = (int32_t)i;
        else if (is_eq && eq_before < need) sel[gt_before + eq_before] = (int32_t)i;
        gt_seen += total & 0xffff;
        eq_seen += total >> 16;
    }
    __syncthreads();                         // sel[] written by this block is read below

    // ---- merge runs of adjacent kept chunks into token spans ----
    int64_t span_base = 0;
    for (int64_t base = 0; base < k; base += kTopkThreads) {
        const int64_t p = base + tid;
        int start = 0, last = 0;
        int32_t c = 0;
        if (p < k) {
            c = sel[p];
            start = (p == 0) || (sel[p - 1] != c - 1);
            last = (p == k - 1) || (sel[p + 1] != c + 1);
        }
        int tot;
        const int id = block_scan_incl(start, wave_tot, tot);            // 1-based span id of this element
        if (p < k) {
            const int64_t s = span_base + id - 1;
            if (start) spans[2 * s] = (int64_t)c * chunk;
            if (last) {
                const int64_t e = ((int64_t)c + 1) * chunk;
                spans[2 * s + 1] = e < L ? e : L;
            }
        }
        span_base += tot;
    }
    if (tid == 0) *n_spans = (int32_t)span_base;
}

template <int R>
__global__ __launch_bounds__(kTopkThreads) void sp_topk_kernel(const float *__restrict__ cs, int64_t n_chunks,
                                                               int64_t k, const int64_t *__restrict__ k_dev,
                                                               int chunk, int64_t L, int32_t *sel,
                                                               int64_t *__restrict__ spans,
                                                               int32_t *__restrict__ n_spans)
{
    topk_body<R>(cs, n_chunks, k, k_dev, chunk, L, sel, spans, n_spans);
}

// Ragged batch: one workgroup per prompt; prompt b keeps k_b = kept_off[b+1] - kept_off[b] chunks and
// writes its indices and spans from kept_off[b] on. An empty prompt keeps nothing.
template <int R>
__global__ __launch_bounds__(kTopkThreads) void sp_topk_batch_kernel(const float *__restrict__ cs,
                                                                     const int64_t *__restrict__ off,
                                                                     const int64_t *__restrict__ kept_off, int chunk,
                                                                     int32_t *sel, int64_t *__restrict__ spans,
                                                                     int32_t *__restrict__ n_spans)
{
    const int b = blockIdx.x;
    const int64_t o = off[b], L = off[b + 1] - o;
    const int64_t n_chunks = (L + chunk - 1) / chunk;
    const int64_t k0 = kept_off[b];
    int64_t k = kept_off[b + 1] - k0;
    if (n_chunks == 0 || k < 1) {            // uniform
        if (threadIdx.x == 0) n_spans[b] = 0;
        return;
    }
    k = k > n_chunks ? n_chunks : k;
    topk_body<R>(cs + batch_chunk_slot(o, b, chunk), n_chunks, k, nullptr, chunk, L, sel + k0, spans + 2 * k0, n_spans + b);
}

// ---------------------------------------------------------------------------
// budget search
// ---------------------------------------------------------------------------
constexpr int kRankThreads = 256;
constexpr int kMaxBudgetChunks = 1 << 16;

// rank[j] = number of chunks that come before chunk j in the order (score descending, index
// ascending). Workgroup (x, y) counts, for the 256 chunks of tile x, the chunks of tile y that come
// before them and adds the counts to rank (cleared beforehand): C^2 comparisons over (C / 256)^2
// workgroups.
__global__ __launch_bounds__(kRankThreads) void sp_rank_kernel(const float *__restrict__ cs, int n_chunks,
                                                               int32_t *__restrict__ rank)
{
    __shared__ uint4 tile[kRankThreads / 4];
    const int j = blockIdx.x * kRankThreads + threadIdx.x;
    const int base = blockIdx.y * kRankThreads;
    const int i = base + threadIdx.x;
    // entries past the last chunk get key 0, the image of no finite score: they never count
    reinterpret_cast<uint32_t *>(tile)[threadIdx.x] = i < n_chunks ? order_key(cs[i]) : 0u;
    __syncthreads();
    if (j >= n_chunks) return;
    const uint32_t mine = order_key(cs[j]);
    int before = 0;
#pragma unroll 4
    for (int t = 0; t < kRankThreads / 4; ++t) {
        const uint4 o = tile[t];
        const int i0 = base + 4 * t;
        before += (o.x > mine) || (o.x == mine && i0 < j);
        before += (o.y > mine) || (o.y == mine && i0 + 1 < j);
        before += (o.z > mine) || (o.z == mine && i0 + 2 < j);
        before += (o.w > mine) || (o.w == mine && i0 + 3 < j);
    }
    if (before) atomicAdd(&rank[j], before);
}

// Character offset of chunk boundary m (0 .. C; boundary C is the end of the text), from the compact
// array the chunk kernel has filled (a few KB: the searches below stay in the caches).
__device__ __forceinline__ int64_t boundary(const int64_t *__restrict__ bnd, int64_t, int, int m) { return bnd[m]; }

// First boundary index in [lo, hi] whose offset is > x (STRICT) or >= x; hi + 1 if none.
template <bool STRICT>
__device__ __forceinline__ int first_boundary(const int64_t *__restrict__ doff, int64_t L, int chunk, int lo, int hi,
                                              int64_t x)
{
    int a = lo, b = hi + 1;
    while (a < b) {
        const int mid = a + ((b - a) >> 1);
        const int64_t e = boundary(doff, L, chunk, mid);
        if (STRICT ? (e > x) : (e >= x)) b = mid; else a = mid + 1;
    }
    return a;
}

__global__ __launch_bounds__(kRankThreads) void sp_token_rank_kernel(const int64_t *__restrict__ doff, int64_t L,
                                                                     int chunk, int n_chunks,
                                                                     const int64_t *__restrict__ toff, int64_t M,
                                                                     const int32_t *__restrict__ rank,
                                                                     int32_t *__restrict__ hist)
{
    const int64_t t = (int64_t)blockIdx.x * kRankThreads + threadIdx.x;
    const bool live = t < M;
    const int64_t a = live ? toff[t] : 0, b = live ? toff[t + 1] : 0;
    const int C = n_chunks;
    int r = C;                                   // bin C: kept by no selection
    if (!live) {
        r = -1;
    } else if (b > a) {
        // chunks j with a < e[j+1] and b > e[j]: a contiguous range
        const int j_lo = first_boundary<true>(doff, L, chunk, 1, C, a) - 1;        // first j with e[j+1] > a
        const int j_hi = first_boundary<false>(doff, L, chunk, 0, C - 1, b) - 1;   // last j with e[j] < b
        if (j_lo < C && j_hi >= 0)
            for (int j = j_lo; j <= j_hi; ++j) r = min(r, rank[j]);
    } else {
        const int m1 = first_boundary<false>(doff, L, chunk, 0, C, a);             // first boundary >= a
        if (m1 <= C && m1 >= 1) {
            if (boundary(doff, L, chunk, m1) != a) {
                r = rank[m1 - 1];                                                   // strictly inside chunk m1 - 1
            } else {
                const int m2 = first_boundary<true>(doff, L, chunk, m1, C, a) - 1;  // last boundary == a
                if (m2 < C) {                    // chunks m1-1 .. m2 all have to be selected
                    int worst = 0;
                    for (int j = m1 - 1; j <= m2; ++j) worst = max(worst, rank[j]);
                    r = worst;
                }
            }
        }
    }
    // Neighbouring tokens mostly share their bin: the first lane of every run of equal r within the
    // wave adds the run's length (integer counts: the histogram is the same in any order).
    const int lane = threadIdx.x & 63;
    const int prev = __shfl_up(r, 1);
    const bool leader = lane == 0 || prev != r;
    const uint64_t leaders = __ballot(leader);
    if (leader && r >= 0) {
        const uint64_t later = lane == 63 ? 0 : leaders >> (lane + 1);
        const int run = later ? __ffsll((unsigned long long)later) : 64 - lane;
        atomicAdd(&hist[r], run);
    }
}

// kept(k) = hist[0] + .. + hist[k-1]; writes the largest k in 1..C with kept(k) <= budget (1 if none)
// and kept at that k.
__global__ __launch_bounds__(kTopkThreads) void sp_budget_kernel(const int32_t *__restrict__ hist, int n_chunks,
                                                                 int64_t budget, int64_t *__restrict__ k_out,
                                                                 int64_t *__restrict__ kept_out)
{
    __shared__ int wave_tot[kTopkThreads / 64];
    __shared__ int s_first;
    const int tid = threadIdx.x;
    int64_t carry = 0, within = 0, kept_within = 0;
    for (int base = 0; base < n_chunks; base += kTopkThreads) {
        const int i = base + tid;
        if (base == 0 && tid == 0) s_first = hist[0];
        const int h = i < n_chunks ? hist[i] : 0;
        int total;
        const int64_t incl = carry + block_scan_incl(h, wave_tot, total);   // kept(i + 1)
        const int ok = (i < n_chunks && incl <= budget) ? 1 : 0;             // a prefix of the k's: kept is monotone
        int ok_total;
        block_scan_incl(ok, wave_tot, ok_total);
        within += ok_total;
        carry += total;
        // kept at the last k within the budget: the largest incl that is <= budget
        int64_t cand = ok ? incl : 0;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const int64_t o = __shfl_xor(cand, off);
            cand = o > cand ? o : cand;
        }
        __shared__ int64_t wave_best[kTopkThreads / 64];
        __syncthreads();
        if ((tid & 63) == 0) wave_best[tid >> 6] = cand;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < kTopkThreads / 64; ++w) kept_within = wave_best[w] > kept_within ? wave_best[w] : kept_within;
    }
    if (tid == 0) {
        *k_out = within >= 1 ? within : 1;
        if (kept_out) *kept_out = within >= 1 ? kept_within : (int64_t)s_first;
    }
}

void launch_topk(hipStream_t st, const float *cs, int64_t C, int64_t k, const int64_t *k_dev, int chunk, int64_t L,
                 int32_t *sel, int64_t *spans, int32_t *n_spans)
{
    const dim3 grid(1), block(kTopkThreads);
    if (C <= 2 * kTopkThreads)
        hipLaunchKernelGGL((sp_topk_kernel<2>), grid, block, 0, st, cs, C, k, k_dev, chunk, L, sel, spans, n_spans);
    else if (C <= 8 * kTopkThreads)
        hipLaunchKernelGGL((sp_topk_kernel<8>), grid, block, 0, st, cs, C, k, k_dev, chunk, L, sel, spans, n_spans);
    else
        hipLaunchKernelGGL((sp_topk_kernel<0>), grid, block, 0, st, cs, C, k, k_dev, chunk, L, sel, spans, n_spans);
}

size_t budget_ws_layout(int64_t C, size_t &off_rank, size_t &off_hist, size_t &off_bnd)
{
    size_t off = sp::align_up(sizeof(float) * (size_t)C, 256);
    off_rank = off; off = sp::align_up(off + sizeof(int32_t) * (size_t)C, 256);
    off_hist = off; off = sp::align_up(off + sizeof(int32_t) * ((size_t)C + 1), 256);
    off_bnd = off;  off = sp::align_up(off + sizeof(int64_t) * ((size_t)C + 1), 256);
    return off;
}

}  // namespace

extern "C" sp_status sp_select_workspace(int64_t L, int32_t chunk, size_t *bytes)
{
    if (!bytes) return sp::fail(SP_ERR_INVALID_ARG, "bytes is null");
    if (L < 1 || chunk < 1) return sp::fail(SP_ERR_INVALID_ARG, "L and chunk must be >= 1");
    const int64_t C = sp::ceil_div(L, chunk);
    *bytes = sp::align_up(sizeof(float) * (size_t)C, 256);
    return SP_OK;
}

namespace {

// Validation shared by the two selection entry points, then the two launches; `cs` receives the chunk scores.
sp_status select_check(const float *scores_dev, int64_t L, int32_t pool_w, int32_t chunk, int64_t k,
                       const int32_t *sel_chunks_dev, const int64_t *spans_dev, const int32_t *n_spans_dev, int64_t &C)
{
    if (!scores_dev || !sel_chunks_dev || !spans_dev || !n_spans_dev)
        return sp::fail(SP_ERR_INVALID_ARG, "scores_dev, sel_chunks_dev, spans_dev and n_spans_dev must not be null");
    if (L < 1) return sp::fail(SP_ERR_INVALID_ARG, "L = %lld must be >= 1", (long long)L);
    if (chunk < 1) return sp::fail(SP_ERR_INVALID_ARG, "chunk = %d must be >= 1", chunk);
    if (pool_w < 1 || pool_w % 2 == 0) return sp::fail(SP_ERR_INVALID_ARG, "pool_w = %d must be odd and >= 1", pool_w);
    if (pool_w > kMaxPool) return sp::fail(SP_ERR_UNSUPPORTED, "pool_w = %d (supported: <= %d)", pool_w, kMaxPool);
    C = sp::ceil_div(L, chunk);
    if (C > (1 << 30)) return sp::fail(SP_ERR_UNSUPPORTED, "too many chunks (%lld)", (long long)C);
    if (k < 1 || k > C) return sp::fail(SP_ERR_INVALID_ARG, "k = %lld outside 1..%lld", (long long)k, (long long)C);
    return SP_OK;
}

sp_status select_launch(const float *scores_dev, int64_t L, int32_t pool_w, int32_t chunk, int64_t k, int64_t C,
                        int32_t *sel_chunks_dev, int64_t *spans_dev, int32_t *n_spans_dev, float *chunk_scores_dev,
                        float *cs, hipStream_t st)
{
    const int waves_per_block = kChunkThreads / 64;
    const unsigned grid = (unsigned)((C + waves_per_block - 1) / waves_per_block);
    hipLaunchKernelGGL(sp_chunk_kernel, dim3(grid), dim3(kChunkThreads), 0, st, scores_dev, L, (int)pool_w,
                       (int)chunk, C, cs, chunk_scores_dev, (const int64_t *)nullptr, (int64_t *)nullptr,
                       (int32_t *)nullptr, (int32_t *)nullptr);
    SP_HIP_CHECK(hipGetLastError());
    launch_topk(st, cs, C, k, nullptr, (int)chunk, L, sel_chunks_dev, spans_dev, n_spans_dev);
    SP_HIP_CHECK(hipGetLastError());
    return SP_OK;
}

}  // namespace

extern "C" sp_status sp_select(const float *scores_dev, int64_t L, int32_t pool_w, int32_t chunk, int64_t k,
                               int32_t *sel_chunks_dev, int64_t *spans_dev, int32_t *n_spans_dev,
                               float *chunk_scores_dev, void *ws_dev, size_t ws_bytes, void *hip_stream)
{
    int64_t C = 0;
    const sp_status rc = select_check(scores_dev, L, pool_w, chunk, k, sel_chunks_dev, spans_dev, n_spans_dev, C);
    if (rc != SP_OK) return rc;
    const size_t need = sp::align_up(sizeof(float) * (size_t)C, 256);
    if (!ws_dev) return sp::fail(SP_ERR_WORKSPACE, "ws_dev is null (%zu bytes needed)", need);
    if ((uintptr_t)ws_dev % 256 != 0) return sp::fail(SP_ERR_WORKSPACE, "ws_dev is not 256-byte aligned");
    if (ws_bytes < need) return sp::fail(SP_ERR_WORKSPACE, "workspace too small: %zu < %zu", ws_bytes, need);
    return select_launch(scores_dev, L, pool_w, chunk, k, C, sel_chunks_dev, spans_dev, n_spans_dev, chunk_scores_dev,
                         static_cast<float *>(ws_dev), static_cast<hipStream_t>(hip_stream));
}

// ---------------------------------------------------------------------------
// sp_select for a ragged batch: two launches for all prompts.
// ---------------------------------------------------------------------------
namespace {
constexpr int kMaxBatchPrompts = 4096;

size_t select_batch_ws(int64_t total, int32_t B, int32_t chunk)
{
    return sp::align_up(sizeof(float) * (size_t)(total / chunk + B + 1), 256);
}
}  // namespace

extern "C" sp_status sp_select_batch_workspace(int64_t total_tokens, int32_t B, int32_t chunk, size_t *bytes)
{
    if (!bytes) return sp::fail(SP_ERR_INVALID_ARG, "bytes is null");
    if (total_tokens < 0 || chunk < 1 || B < 1 || B > kMaxBatchPrompts)
        return sp::fail(SP_ERR_INVALID_ARG, "total_tokens >= 0, chunk >= 1 and B in 1..%d are required", kMaxBatchPrompts);
    if (total_tokens / chunk > (int64_t(1) << 42))       // 4096 prompts of 2^30 chunks: what sp_select_batch accepts at most
        return sp::fail(SP_ERR_UNSUPPORTED, "too many chunks (%lld)", (long long)(total_tokens / chunk));
    *bytes = select_batch_ws(total_tokens, B, chunk);
    return SP_OK;
}

extern "C" sp_status sp_select_batch(const float *scores_dev, const int64_t *offsets_host, const int64_t *offsets_dev,
                                     int32_t B, int32_t pool_w, int32_t chunk, const int64_t *kept_off_host,
                                     const int64_t *kept_off_dev, int32_t *sel_chunks_dev, int64_t *spans_dev,
                                     int32_t *n_spans_dev, float *chunk_scores_dev, void *ws_dev, size_t ws_bytes,
                                     void *hip_stream)
{
    if (!scores_dev || !offsets_host || !offsets_dev || !kept_off_host || !kept_off_dev || !sel_chunks_dev || !spans_dev ||
        !n_spans_dev)
        return sp::fail(SP_ERR_INVALID_ARG, "only chunk_scores_dev may be null");
    if (B < 1 || B > kMaxBatchPrompts) return sp::fail(SP_ERR_INVALID_ARG, "B = %d (supported: 1..%d)", B, kMaxBatchPrompts);
    if (chunk < 1) return sp::fail(SP_ERR_INVALID_ARG, "chunk = %d must be >= 1", chunk);
    if (pool_w < 1 || pool_w % 2 == 0) return sp::fail(SP_ERR_INVALID_ARG, "pool_w = %d must be odd and >= 1", pool_w);
    if (pool_w > kMaxPool) return sp::fail(SP_ERR_UNSUPPORTED, "pool_w = %d (supported: <= %d)", pool_w, kMaxPool);
    if (offsets_host[0] != 0 || kept_off_host[0] != 0)
        return sp::fail(SP_ERR_INVALID_ARG, "offsets_host[0] and kept_off_host[0] must be 0");
    int64_t max_chunks = 0;
    for (int b = 0; b < B; ++b) {
        const int64_t len = offsets_host[b + 1] - offsets_host[b], k = kept_off_host[b + 1] - kept_off_host[b];
        if (len < 0) return sp::fail(SP_ERR_INVALID_ARG, "offsets_host decreases at prompt %d", b);
        const int64_t C = sp::ceil_div(len, chunk);
        if (C > (1 << 30)) return sp::fail(SP_ERR_UNSUPPORTED, "too many chunks (%lld) in prompt %d", (long long)C, b);
        if (len == 0 ? k != 0 : (k < 1 || k > C))
            return sp::fail(SP_ERR_INVALID_ARG, "prompt %d keeps %lld chunks of %lld (1..C, or 0 of an empty prompt)", b,
                            (long long)k, (long long)C);
        max_chunks = std::max(max_chunks, C);
    }
    const size_t need = select_batch_ws(offsets_host[B], B, chunk);
    if (!ws_dev) return sp::fail(SP_ERR_WORKSPACE, "ws_dev is null (%zu bytes needed)", need);
    if ((uintptr_t)ws_dev % 256 != 0) return sp::fail(SP_ERR_WORKSPACE, "ws_dev is not 256-byte aligned");
    if (ws_bytes < need) return sp::fail(SP_ERR_WORKSPACE, "workspace too small: %zu < %zu", ws_bytes, need);
    if (max_chunks == 0) max_chunks = 1;     // all prompts empty: the top-k launch still writes n_spans = 0
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    float *cs = static_cast<float *>(ws_dev);
    const int waves_per_block = kChunkThreads / 64;
    hipLaunchKernelGGL(sp_chunk_batch_kernel, dim3((unsigned)sp::ceil_div(max_chunks, waves_per_block), (unsigned)B),
                       dim3(kChunkThreads), 0, st, scores_dev, offsets_dev, (int)pool_w, (int)chunk, cs, chunk_scores_dev);
    SP_HIP_CHECK(hipGetLastError());
    const dim3 grid((unsigned)B), block(kTopkThreads);
    if (max_chunks <= 2 * kTopkThreads)
        hipLaunchKernelGGL((sp_topk_batch_kernel<2>), grid, block, 0, st, cs, offsets_dev, kept_off_dev, (int)chunk,
                           sel_chunks_dev, spans_dev, n_spans_dev);
    else if (max_chunks <= 8 * kTopkThreads)
        hipLaunchKernelGGL((sp_topk_batch_kernel<8>), grid, block, 0, st, cs, offsets_dev, kept_off_dev, (int)chunk,
                           sel_chunks_dev, spans_dev, n_spans_dev);
    else
        hipLaunchKernelGGL((sp_topk_batch_kernel<0>), grid, block, 0, st, cs, offsets_dev, kept_off_dev, (int)chunk,
                           sel_chunks_dev, spans_dev, n_spans_dev);
    SP_HIP_CHECK(hipGetLastError());
    return SP_OK;
}

// ---------------------------------------------------------------------------
// sp_select without a workspace argument, for callers that cannot allocate: the
// chunk scores go to a device array that is part of the library's image.
// ---------------------------------------------------------------------------
constexpr int64_t kStaticChunks = SP_SELECT_STATIC_MAX_CHUNKS;
static __device__ __align__(256) float scratch[kStaticChunks];

namespace {

constexpr int kMaxDevices = 64;
// Device address of `scratch` on each device, resolved once per device with that device current.
// (In host code the array's name only stands for the symbol; it is not a device address.)
std::atomic<float *> g_scratch[kMaxDevices];

sp_status scratch_of_current_device(float *&out)
{
    int dev = -1;
    SP_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return sp::fail(SP_ERR_UNSUPPORTED, "device index %d (supported: < %d)", dev, kMaxDevices);
    float *p = g_scratch[dev].load(std::memory_order_acquire);
    if (!p) {
        void *sym = nullptr;
        SP_HIP_CHECK(hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)));
        if (!sym) return sp::fail(SP_ERR_DEVICE, "the library's scratch array has no address on device %d", dev);
        p = static_cast<float *>(sym);
        g_scratch[dev].store(p, std::memory_order_release);     // every thread resolves the same address
    }
    out = p;
    return SP_OK;
}

}  // namespace

extern "C" sp_status sp_select_static(const float *scores_dev, int64_t L, int32_t pool_w, int32_t chunk, int64_t k,
                                      int32_t *sel_chunks_dev, int64_t *spans_dev, int32_t *n_spans_dev,
                                      float *chunk_scores_dev, void *hip_stream)
{
    int64_t C = 0;
    const sp_status rc = select_check(scores_dev, L, pool_w, chunk, k, sel_chunks_dev, spans_dev, n_spans_dev, C);
    if (rc != SP_OK) return rc;
    if (C > kStaticChunks)
        return sp::fail(SP_ERR_UNSUPPORTED, "%lld chunks exceed the %lld the library's own scratch array holds; use sp_select",
                        (long long)C, (long long)kStaticChunks);
    float *cs = nullptr;
    const sp_status rs = scratch_of_current_device(cs);
    if (rs != SP_OK) return rs;
    // every chunk score the top-k kernel reads is written by the chunk kernel of this call: nothing to clear
    return select_launch(scores_dev, L, pool_w, chunk, k, C, sel_chunks_dev, spans_dev, n_spans_dev, chunk_scores_dev, cs,
                         static_cast<hipStream_t>(hip_stream));
}

extern "C" sp_status sp_select_budget_workspace(int64_t L, int32_t chunk, size_t *bytes)
{
    if (!bytes) return sp::fail(SP_ERR_INVALID_ARG, "bytes is null");
    if (L < 1 || chunk < 1) return sp::fail(SP_ERR_INVALID_ARG, "L and chunk must be >= 1");
    const int64_t C = sp::ceil_div(L, chunk);
    if (C > kMaxBudgetChunks)
        return sp::fail(SP_ERR_UNSUPPORTED, "%lld chunks (the budget search supports <= %d)", (long long)C, kMaxBudgetChunks);
    size_t a, b, c;
    *bytes = budget_ws_layout(C, a, b, c);
    return SP_OK;
}

extern "C" sp_status sp_select_budget(const float *scores_dev, int64_t L, int32_t pool_w, int32_t chunk,
                                      const int64_t *draft_off_dev, const int64_t *target_off_dev, int64_t M,
                                      int64_t budget, int32_t *sel_chunks_dev, int64_t *spans_dev,
                                      int32_t *n_spans_dev, int64_t *k_dev, int64_t *n_kept_dev,
                                      float *chunk_scores_dev, void *ws_dev, size_t ws_bytes, void *hip_stream)
{
    if (!scores_dev || !draft_off_dev || !target_off_dev || !sel_chunks_dev || !spans_dev || !n_spans_dev || !k_dev)
        return sp::fail(SP_ERR_INVALID_ARG, "only n_kept_dev and chunk_scores_dev may be null");
    if (L < 1 || M < 1) return sp::fail(SP_ERR_INVALID_ARG, "L = %lld and M = %lld must be >= 1", (long long)L, (long long)M);
    if (chunk < 1) return sp::fail(SP_ERR_INVALID_ARG, "chunk = %d must be >= 1", chunk);
    if (pool_w < 1 || pool_w % 2 == 0) return sp::fail(SP_ERR_INVALID_ARG, "pool_w = %d must be odd and >= 1", pool_w);
    if (pool_w > kMaxPool) return sp::fail(SP_ERR_UNSUPPORTED, "pool_w = %d (supported: <= %d)", pool_w, kMaxPool);
    if (budget < 0) return sp::fail(SP_ERR_INVALID_ARG, "budget = %lld is negative", (long long)budget);
    if (M >= (int64_t(1) << 31)) return sp::fail(SP_ERR_UNSUPPORTED, "M = %lld (supported: < 2^31)", (long long)M);
    const int64_t C = sp::ceil_div(L, chunk);
    if (C > kMaxBudgetChunks)
        return sp::fail(SP_ERR_UNSUPPORTED, "%lld chunks (the budget search supports <= %d)", (long long)C, kMaxBudgetChunks);
    size_t off_rank, off_hist, off_bnd;
    const size_t need = budget_ws_layout(C, off_rank, off_hist, off_bnd);
    if (!ws_dev) return sp::fail(SP_ERR_WORKSPACE, "ws_dev is null (%zu bytes needed)", need);
    if ((uintptr_t)ws_dev % 256 != 0) return sp::fail(SP_ERR_WORKSPACE, "ws_dev is not 256-byte aligned");
    if (ws_bytes < need) return sp::fail(SP_ERR_WORKSPACE, "workspace too small: %zu < %zu", ws_bytes, need);

    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char *ws = static_cast<char *>(ws_dev);
    float *cs = reinterpret_cast<float *>(ws);
    int32_t *rank = reinterpret_cast<int32_t *>(ws + off_rank);
    int32_t *hist = reinterpret_cast<int32_t *>(ws + off_hist);
    int64_t *bnd = reinterpret_cast<int64_t *>(ws + off_bnd);
    const int waves_per_block = kChunkThreads / 64;
    hipLaunchKernelGGL(sp_chunk_kernel, dim3((unsigned)((C + waves_per_block - 1) / waves_per_block)),
                       dim3(kChunkThreads), 0, st, scores_dev, L, (int)pool_w, (int)chunk, C, cs, chunk_scores_dev,
                       draft_off_dev, bnd, rank, hist);
    SP_HIP_CHECK(hipGetLastError());
    const unsigned n_tiles = (unsigned)((C + kRankThreads - 1) / kRankThreads);
    hipLaunchKernelGGL(sp_rank_kernel, dim3(n_tiles, n_tiles), dim3(kRankThreads), 0, st, (const float *)cs, (int)C, rank);
    SP_HIP_CHECK(hipGetLastError());
    hipLaunchKernelGGL(sp_token_rank_kernel, dim3((unsigned)((M + kRankThreads - 1) / kRankThreads)), dim3(kRankThreads),
                       0, st, (const int64_t *)bnd, L, (int)chunk, (int)C, target_off_dev, M, (const int32_t *)rank, hist);
    SP_HIP_CHECK(hipGetLastError());
    hipLaunchKernelGGL(sp_budget_kernel, dim3(1), dim3(kTopkThreads), 0, st, (const int32_t *)hist, (int)C, budget, k_dev,
                       n_kept_dev);
    SP_HIP_CHECK(hipGetLastError());
    launch_topk(st, cs, C, 1, k_dev, (int)chunk, L, sel_chunks_dev, spans_dev, n_spans_dev);
    SP_HIP_CHECK(hipGetLastError());
    return SP_OK;
}

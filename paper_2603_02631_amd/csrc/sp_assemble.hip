// sp_assemble: token ids and position ids of the compressed target prompt
// (paper: Algorithm 1 "ConcatWithDelim", the target tokenisation of the
// compressed text and the new contiguous position ids; Section 3.2).
//
// The kept target ranges are copied in order with the delimiter's ids between
// consecutive ranges. Range r occupies one block of the output: its delimiter
// (for r > 0) followed by its tokens.
//
//   sp_assemble_offsets_kernel  one workgroup: exclusive prefix sum of the block
//                               lengths -> block starts (workspace), total length.
//   sp_assemble_gather_kernel   one thread per output entry: binary search of the
//                               block starts, then a delimiter id or a token id.
#include "sp_common.hpp"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

__device__ __forceinline__ int64_t clamp64(int64_t v, int64_t lo, int64_t hi) { return v < lo ? lo : (v > hi ? hi : v); }

__global__ __launch_bounds__(kThreads) void sp_assemble_offsets_kernel(const int64_t *__restrict__ tspans,
                                                                       const int32_t *__restrict__ n_tspans_p,
                                                                       int max_spans, int64_t M, int n_delim,
                                                                       int64_t *__restrict__ block_start,
                                                                       int64_t *__restrict__ out_len)
{
    __shared__ int64_t wave_tot[kWaves];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int n = *n_tspans_p;
    n = n < 0 ? 0 : (n > max_spans ? max_spans : n);
    int64_t carry = 0;
    for (int base = 0; base < n; base += kThreads) {
        const int r = base + tid;
        int64_t len = 0;
        if (r < n) {
            const int64_t b = clamp64(tspans[2 * r], 0, M), e = clamp64(tspans[2 * r + 1], b, M);
            len = (e - b) + (r > 0 ? n_delim : 0);
        }
        int64_t x = len;                    // inclusive scan within the wave
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int64_t y = __shfl_up(x, off);
            if (lane >= off) x += y;
        }
        __syncthreads();                    // wave_tot of the previous segment has been read
        if (lane == 63) wave_tot[wave] = x;
        __syncthreads();
        int64_t before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            if (w < wave) before += wave_tot[w];
            total += wave_tot[w];
        }
        if (r < n) block_start[r] = carry + before + x - len;
        carry += total;
    }
    if (tid == 0) {
        block_start[n] = carry;             // sentinel: one past the last block
        *out_len = carry;
    }
}

__global__ __launch_bounds__(kThreads) void sp_assemble_gather_kernel(const int32_t *__restrict__ target_ids, int64_t M,
                                                                      const int64_t *__restrict__ tspans,
                                                                      const int32_t *__restrict__ n_tspans_p,
                                                                      int max_spans,
                                                                      const int32_t *__restrict__ delim, int n_delim,
                                                                      const int64_t *__restrict__ block_start,
                                                                      int64_t out_capacity, int32_t *__restrict__ out_ids,
                                                                      int32_t *__restrict__ out_pos,
                                                                      int64_t *__restrict__ out_src)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    int n = *n_tspans_p;
    n = n < 0 ? 0 : (n > max_spans ? max_spans : n);
    const int64_t total = block_start[n];
    if (i >= total || i >= out_capacity) return;
    // last block whose start is <= i
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = lo + ((hi - lo) >> 1);
        if (block_start[mid] <= i) lo = mid + 1; else hi = mid;
    }
    const int r = lo - 1;
    int64_t j = i - block_start[r];
    int32_t id;
    int64_t src;
    if (r > 0 && j < n_delim) {
        id = delim[j];
        src = -1;
    } else {
        if (r > 0) j -= n_delim;
        src = clamp64(tspans[2 * r], 0, M) + j;
        id = target_ids[src];
    }
    out_ids[i] = id;
    out_pos[i] = (int32_t)i;
    if (out_src) out_src[i] = src;
}

size_t workspace_need(int32_t max_spans) { return sp::align_up(sizeof(int64_t) * ((size_t)max_spans + 1), 256); }

}  // namespace

extern "C" sp_status sp_assemble_workspace(int32_t max_spans, size_t *bytes)
{
    if (!bytes) return sp::fail(SP_ERR_INVALID_ARG, "bytes is null");
    if (max_spans < 1 || max_spans > (1 << 24))
        return sp::fail(SP_ERR_INVALID_ARG, "max_spans = %d outside 1..2^24", max_spans);
    *bytes = workspace_need(max_spans);
    return SP_OK;
}

extern "C" sp_status sp_assemble(const int32_t *target_ids_dev, int64_t M, const int64_t *tspans_dev,
                                 const int32_t *n_tspans_dev, int32_t max_spans, const int32_t *delim_ids_dev,
                                 int32_t n_delim, int64_t out_capacity, int32_t *out_ids_dev, int32_t *out_pos_dev,
                                 int64_t *out_src_dev, int64_t *out_len_dev, void *ws_dev, size_t ws_bytes,
                                 void *hip_stream)
{
    if (!target_ids_dev || !tspans_dev || !n_tspans_dev || !out_ids_dev || !out_pos_dev || !out_len_dev)
        return sp::fail(SP_ERR_INVALID_ARG, "only delim_ids_dev (with n_delim = 0) and out_src_dev may be null");
    if (M < 1) return sp::fail(SP_ERR_INVALID_ARG, "M = %lld must be >= 1", (long long)M);
    if (max_spans < 1 || max_spans > (1 << 24))
        return sp::fail(SP_ERR_INVALID_ARG, "max_spans = %d outside 1..2^24", max_spans);
    if (n_delim < 0 || n_delim > 1024) return sp::fail(SP_ERR_INVALID_ARG, "n_delim = %d outside 0..1024", n_delim);
    if (n_delim > 0 && !delim_ids_dev) return sp::fail(SP_ERR_INVALID_ARG, "delim_ids_dev is null with n_delim = %d", n_delim);
    if (out_capacity < 1 || out_capacity >= (int64_t(1) << 31))
        return sp::fail(SP_ERR_INVALID_ARG, "out_capacity = %lld outside 1..2^31-1", (long long)out_capacity);
    const size_t need = workspace_need(max_spans);
    if (!ws_dev) return sp::fail(SP_ERR_WORKSPACE, "ws_dev is null (%zu bytes needed)", need);
    if ((uintptr_t)ws_dev % 256 != 0) return sp::fail(SP_ERR_WORKSPACE, "ws_dev is not 256-byte aligned");
    if (ws_bytes < need) return sp::fail(SP_ERR_WORKSPACE, "workspace too small: %zu < %zu", ws_bytes, need);

    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    int64_t *block_start = static_cast<int64_t *>(ws_dev);
    hipLaunchKernelGGL(sp_assemble_offsets_kernel, dim3(1), dim3(kThreads), 0, st, tspans_dev, n_tspans_dev,
                       (int)max_spans, M, (int)n_delim, block_start, out_len_dev);
    SP_HIP_CHECK(hipGetLastError());
    // the output cannot be longer than every target token plus a delimiter per range
    int64_t bound = M + (int64_t)(max_spans - 1) * n_delim;
    if (bound > out_capacity) bound = out_capacity;
    const unsigned grid = (unsigned)((bound + kThreads - 1) / kThreads);
    hipLaunchKernelGGL(sp_assemble_gather_kernel, dim3(grid), dim3(kThreads), 0, st, target_ids_dev, M, tspans_dev,
                       n_tspans_dev, (int)max_spans, delim_ids_dev, (int)n_delim, (const int64_t *)block_start,
                       out_capacity, out_ids_dev, out_pos_dev, out_src_dev);
    SP_HIP_CHECK(hipGetLastError());
    return SP_OK;
}

// sp_score / sp_score_batch: token importance from the lookahead queries'
// attention over the prompt keys (paper: Appendix A.1.1; Algorithm 1,
// "AggregateMaxMean").
//
// Three kernels, all built around the bf16 32x32x16 MFMA of gfx950:
//   stats   one workgroup per (key tile, layer, kv head): logits of the kv
//           head's whole query group against 256 keys, per-row running
//           (max, sum of exp) kept per lane, one partial per (row, tile);
//   merge   log-sum-exp combination of the partials of each row in a fixed
//           order (deterministic), giving the row's normaliser;
//   prob    one workgroup per (key tile, layer range), looping over its layers
//           and the kv heads:
//           logits again with the normaliser folded into the MFMA's C operand,
//           maximum over heads taken on logits (exp is monotone, so
//           max_h softmax_h = exp(max_h(logit_h - lse_h))), one exp per
//           (lookahead row, key), sum over lookahead rows and layers in
//           registers, a single store per key. Long inputs give every
//           workgroup all layers; short ones split the layers over several
//           workgroups per tile, which leave per-range results that a fourth
//           kernel (reduce) combines in a fixed order.
//
// Register/lane layout facts used throughout (v_mfma_f32_32x32x16_bf16):
//   A operand: lane i holds row i%32, eight consecutive k-values of half i/32
//   B operand: lane i holds column i%32, the same eight k-values
//   D: lane i, register r holds row 8*(r/4) + 4*(i/32) + r%4, column i%32.
// Since A and B fragments are laid out alike, one fragment of K serves as A
// (rows = keys) in the stats pass and as B (columns = keys) in the prob pass.
#include "sp_common.hpp"
#include "sp_score_dev.hpp"
#include "sp_score_fused.hpp"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

namespace {

using namespace sp_dev;

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kMaxPrompts = 4096;
constexpr size_t kLdsBudget = 64 * 1024;
constexpr int kProbTargetWgs = 1024;   // the prob pass splits layers until it has about this many workgroups

struct TileInfo {
    int64_t j0;          // first key of the tile (index into the packed token axis)
    int64_t end;         // one past the last key of the tile's prompt
    int32_t prompt;
    int32_t first_tile;  // index of the prompt's first tile
};

struct ScoreArgs {
    const uint16_t *q;        // [B][Lyr][H][n_q][d]
    int64_t k_stride_token, k_stride_head;
    const TileInfo *tiles;    // null: single prompt, tile t starts at t * tile_keys
    const int32_t *prompt_tiles;  // [B+1] first tile of each prompt (batch only)
    int64_t L;                // single prompt length
    float2 *part;             // [n_phases][n_tiles][rows_pad]
    float *lse_neg;           // [B][n_phases][rows_pad]  (-lse in raw-logit units, permuted)
    float *scores;
    uint32_t *status;         // the call's status word (cleared here: this path cannot give up)
    const int32_t *block_table;   // paged keys (single prompt): token j lives in page block_table[j / page_tokens]
    int64_t page_tokens;          // of its layer's pool, page p at element offset p * page_stride; null: contiguous
    int64_t page_stride;
    const float *look;        // [n_phases][rows_pad] lookahead-key term of each row's normaliser, or null
    const float *kscale;      // 8-bit keys: [n_phases] scale of each (layer, kv head); null: bf16 keys
    float *split_buf;         // layer-split results: MEAN [n_splits][n_tiles][TILE],
                              //                      MAX  [n_splits][8*n_nblk][n_tiles][TILE]
    int32_t n_splits, layers_per_split;
    int32_t n_tiles, n_prompts;
    int32_t n_layers, n_q_heads, n_kv_heads, group, n_q;
    int32_t n_nblk, n_gblk, rows_pad;   // blocks of 8 lookahead rows / 4 group heads
    int32_t layer_agg;
    float c;                  // scale * log2(e)
    float inv_c;
    float out_scale;          // 1/n_q or 1/(n_q * Lyr)
};

__device__ __forceinline__ TileInfo get_tile(const ScoreArgs &a, int tile, int tile_keys)
{
    if (a.tiles) return a.tiles[tile];
    TileInfo t;
    t.j0 = (int64_t)tile * tile_keys;
    t.end = a.L;
    t.prompt = 0;
    t.first_tile = 0;
    return t;
}

// Address of key 0 of the tile's address space in (layer, kv head): the layer's buffer for contiguous
// keys; for paged keys the tile's page, moved back by the page's first token so that the absolute key
// index still applies (tiles never straddle pages: a page holds a multiple of the tile size).
__device__ __forceinline__ const uint16_t *key_base(const ScoreArgs &a, const LayerPtrs &kp, int layer, int kv,
                                                    const TileInfo &ti)
{
    const uint16_t *b = kp.p[layer] + (int64_t)kv * a.k_stride_head;
    if (a.block_table) {
        const int64_t page = ti.j0 / a.page_tokens;
        b += (int64_t)a.block_table[page] * a.page_stride - page * a.page_tokens * a.k_stride_token;
    }
    return b;
}

// Padded query-row order of one kv head's group: row = blk*32 + rho with
// blk = gblk * n_nblk + nblk, rho = 8*gl + nl  ->  group head g = 4*gblk + gl,
// lookahead row n = 8*nblk + nl. In the D layout of the prob pass this puts the
// four group heads of a block in registers r/4 of one lane.
__device__ __forceinline__ bool row_to_gn(const ScoreArgs &a, int row, int &g, int &n)
{
    const int blk = row >> 5, rho = row & 31;
    const int gblk = blk / a.n_nblk, nblk = blk - gblk * a.n_nblk;
    g = 4 * gblk + (rho >> 3);
    n = 8 * nblk + (rho & 7);
    return g < a.group && n < a.n_q;
}

// 8-bit keys (contiguous only): byte address of key 0 of (layer, kv head).
__device__ __forceinline__ const uint8_t *key_base_fp8(const ScoreArgs &a, const LayerPtrs &kp, int layer, int kv)
{
    return reinterpret_cast<const uint8_t *>(kp.p[layer]) + (int64_t)kv * a.k_stride_head;
}

template <int D>
__device__ __forceinline__ void stage_q(u32x4 *qs, const ScoreArgs &a, int prompt, int layer, int kv, int tid)
{
    constexpr int CH = D / 8;
    const uint16_t *qb = a.q + (((int64_t)prompt * a.n_layers + layer) * a.n_q_heads + (int64_t)kv * a.group) *
                                   a.n_q * D;
    for (int i = tid; i < a.rows_pad * CH; i += kThreads) {
        const int row = i / CH, ch = i - row * CH;
        int g, n;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (row_to_gn(a, row, g, n))
            v = *reinterpret_cast<const u32x4 *>(qb + ((int64_t)g * a.n_q + n) * D + ch * 8);
        qs[lds_slot<D>(row, ch)] = v;
    }
}

// The same staging for 8-bit keys: kb8 addresses bytes, strides are in elements (= bytes).
template <int D, int NS>
__device__ __forceinline__ void stage_k_fp8(u32x4 *ks, const uint8_t *kb8, int64_t stride_token, int64_t j0,
                                            int64_t end, int tid)
{
    constexpr int CH = D / 8;
    constexpr int TILE = kWaves * NS * 32;
    constexpr int N = TILE * CH / kThreads;
    uint2 v[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int idx = tid + i * kThreads;
        const int row = idx / CH, ch = idx % CH;
        const int64_t j = j0 + row;
        v[i] = *reinterpret_cast<const uint2 *>(kb8 + (j < end ? j : end - 1) * stride_token + ch * 8);
    }
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int idx = tid + i * kThreads;
        ks[lds_slot<D>(idx / CH, idx % CH)] = e4m3x8_to_bf16x8(v[i].x, v[i].y);
    }
}

template <int D, int NS>
__device__ __forceinline__ void stage_k(u32x4 *ks, const uint16_t *kb, int64_t stride_token, int64_t j0,
                                        int64_t end, int tid)
{
    constexpr int CH = D / 8;
    constexpr int TILE = kWaves * NS * 32;
    constexpr int N = TILE * CH / kThreads;
    u32x4 v[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int idx = tid + i * kThreads;
        const int row = idx / CH, ch = idx % CH;
        const int64_t j = j0 + row;
        // rows past the end repeat the last key (every consumer masks them): unconditional loads keep
        // the register count a third of what per-load branches cost
        v[i] = *reinterpret_cast<const u32x4 *>(kb + (j < end ? j : end - 1) * stride_token + ch * 8);
    }
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int idx = tid + i * kThreads;
        ks[lds_slot<D>(idx / CH, idx % CH)] = v[i];
    }
}

// ---------------------------------------------------------------------------
// stats: partial (max, sum exp) of every query row of one (layer, kv head)
// over one key tile.
// ---------------------------------------------------------------------------
template <int D, int NS, bool FP8>
__global__ __launch_bounds__(kThreads, 4) void sp_stats_kernel(ScoreArgs a, LayerPtrs kp)
{
    constexpr int KS = D / 16;
    constexpr int TILE = kWaves * NS * 32;
    extern __shared__ u32x4 lds[];
    u32x4 *ks = lds;                         // TILE rows
    u32x4 *qs = lds + TILE * (D / 8);        // rows_pad rows
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, hf = lane >> 5, col = lane & 31;
    const int tile = blockIdx.x, phase = blockIdx.y;
    const int layer = phase / a.n_kv_heads, kv = phase - layer * a.n_kv_heads;
    const TileInfo ti = get_tile(a, tile, TILE);
    if (tile == 0 && phase == 0 && tid == 0) *a.status = 0u;

    stage_q<D>(qs, a, ti.prompt, layer, kv, tid);
    if (FP8) stage_k_fp8<D, NS>(ks, key_base_fp8(a, kp, layer, kv), a.k_stride_token, ti.j0, ti.end, tid);
    else stage_k<D, NS>(ks, key_base(a, kp, layer, kv, ti), a.k_stride_token, ti.j0, ti.end, tid);
    __syncthreads();

    bf16x8 kf[NS][KS];
#pragma unroll
    for (int s = 0; s < NS; ++s) load_frag<D>(ks, (wave * NS + s) * 32 + col, hf, kf[s]);
    __syncthreads();                         // ks is reused for the per-wave statistics below
    float2 *wstats = reinterpret_cast<float2 *>(ks);   // [kWaves][rows_pad]

    // statistics are kept in units of the raw dot product with the stored keys; with 8-bit keys the
    // (layer, kv head)'s scale joins the logit scale
    const float c = FP8 ? a.c * a.kscale[phase] : a.c;
    const int n_blk = a.rows_pad >> 5;
    for (int blk = 0; blk < n_blk; ++blk) {
        bf16x8 qf[KS];
        load_frag<D>(qs, blk * 32 + col, hf, qf);
        float m = neg_inf(), l = 0.f;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            f32x16 acc = {0.f};
#pragma unroll
            for (int t = 0; t < KS; ++t) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s][t], qf[t], acc, 0, 0, 0);
            // acc[r]: key (wave*NS+s)*32 + 8*(r/4) + 4*hf + r%4 of the tile, query row blk*32 + col
            const int64_t left = ti.end - (ti.j0 + (wave * NS + s) * 32);
            if (left >= 32) {
                float tm = acc[0];
#pragma unroll
                for (int r = 1; r < 16; ++r) tm = fmaxf(tm, acc[r]);
                const float mn = fmaxf(m, tm);
                l *= fast_exp2((m - mn) * c);
                m = mn;
                const float mc = mn * c;
                float sum = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) sum += fast_exp2(fmaf(acc[r], c, -mc));
                l += sum;
            } else if (left > 0) {
                float tm = neg_inf();
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = 8 * (r >> 2) + 4 * hf + (r & 3);
                    if (key < left) tm = fmaxf(tm, acc[r]);
                }
                if (tm > neg_inf()) {
                    const float mn = fmaxf(m, tm);
                    l *= fast_exp2((m - mn) * c);
                    m = mn;
                    const float mc = mn * c;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = 8 * (r >> 2) + 4 * hf + (r & 3);
                        if (key < left) l += fast_exp2(fmaf(acc[r], c, -mc));
                    }
                }
            }
        }
        const float m2 = __shfl_xor(m, 32), l2 = __shfl_xor(l, 32);
        lse_merge(m, l, m2, l2, c);
        if (hf == 0) wstats[wave * a.rows_pad + blk * 32 + col] = make_float2(m, l);
    }
    __syncthreads();
    for (int row = tid; row < a.rows_pad; row += kThreads) {
        float2 s0 = wstats[row];
        float m = s0.x, l = s0.y;
#pragma unroll
        for (int w = 1; w < kWaves; ++w) {
            const float2 sw = wstats[w * a.rows_pad + row];
            lse_merge(m, l, sw.x, sw.y, c);
        }
        a.part[((int64_t)phase * a.n_tiles + tile) * a.rows_pad + row] = make_float2(m, l);
    }
}

// ---------------------------------------------------------------------------
// merge: one workgroup per (32-row block, phase, prompt). 8 slices of the
// prompt's tiles are reduced by 32 thread groups, then combined in slice order.
// Writes -lse in raw-logit units, i.e. -(m + log2(l)/c), at the position the
// prob pass reads it from: within a block, row rho = 8*q + 4*hf + e goes to
// hf*16 + 4*q + e. Padding rows get -inf so they never win a maximum.
// ---------------------------------------------------------------------------
constexpr int kMergeSlices = 32;             // thread groups of 32 rows that share a prompt's tiles
constexpr int kMergeThreads = 32 * kMergeSlices;

__global__ __launch_bounds__(kMergeThreads) void sp_merge_kernel(ScoreArgs a)
{
    __shared__ float2 red[kMergeSlices][32];
    const int tid = threadIdx.x, rho = tid & 31, slice = tid >> 5;
    const int blk = blockIdx.x, phase = blockIdx.y, prompt = blockIdx.z;
    const int n_phases = a.n_layers * a.n_kv_heads;
    int t0 = 0, t1 = a.n_tiles;
    if (a.prompt_tiles) { t0 = a.prompt_tiles[prompt]; t1 = a.prompt_tiles[prompt + 1]; }
    const int row = blk * 32 + rho;
    const float c = a.kscale ? a.c * a.kscale[phase] : a.c;      // the phase's logit scale (8-bit keys carry their own)
    const float inv_c = a.kscale ? 1.0f / c : a.inv_c;
    float m = neg_inf(), l = 0.f;
    for (int t = t0 + slice; t < t1; t += kMergeSlices) {
        const float2 p = a.part[((int64_t)phase * a.n_tiles + t) * a.rows_pad + row];
        lse_merge(m, l, p.x, p.y, c);
    }
    red[slice][rho] = make_float2(m, l);
    __syncthreads();
    if (slice == 0) {
#pragma unroll
        for (int s = 1; s < kMergeSlices; ++s) lse_merge(m, l, red[s][rho].x, red[s][rho].y, c);
        int g, n;
        const bool valid = row_to_gn(a, row, g, n) && l > 0.f;
        float v = valid ? -(m + fast_log2(l) * inv_c) : neg_inf();
        if (valid && a.look != nullptr) {
            // the softmax also runs over the row's visible lookahead keys: log-sum-exp of both parts
            const float lp = -v, lk = a.look[(int64_t)phase * a.rows_pad + row], top = fmaxf(lp, lk);
            v = -(top + fast_log2(fast_exp2((lp - top) * a.c) + fast_exp2((lk - top) * a.c)) * a.inv_c);
        }
        const int pos = ((rho >> 2) & 1) * 16 + 4 * (rho >> 3) + (rho & 3);
        a.lse_neg[((int64_t)prompt * n_phases + phase) * a.rows_pad + blk * 32 + pos] = v;
    }
}

// ---------------------------------------------------------------------------
// look: log-sum-exp (raw-logit units) of every query row over the lookahead
// keys it sees, one workgroup per (layer, kv head), one thread per padded row.
// Lookahead row n sees the keys of rows 0 .. n-1, and its own with look_self
// (a decode step attends to the tokens generated before it; Algorithm 1's
// ForwardWithAttn with lookahead = i). Rows that see none get -inf.
// k_look is dense [Lyr][Hkv][n_q][d].
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void sp_look_kernel(ScoreArgs a, const uint16_t *__restrict__ k_look,
                                                           int look_self, int D, float *__restrict__ out)
{
    const int phase = blockIdx.x, row = threadIdx.x;
    if (row >= a.rows_pad) return;
    const int layer = phase / a.n_kv_heads, kv = phase - layer * a.n_kv_heads;
    int g, n;
    float v = neg_inf();
    if (row_to_gn(a, row, g, n)) {
        const uint16_t *qr = a.q + (((int64_t)layer * a.n_q_heads + (int64_t)kv * a.group + g) * a.n_q + n) * D;
        const uint16_t *kb = k_look + ((int64_t)layer * a.n_kv_heads + kv) * a.n_q * D;
        const int n_vis = min(n + (look_self ? 1 : 0), a.n_q);
        float m = neg_inf(), l = 0.f;
        for (int j = 0; j < n_vis; ++j) {
            float dot = 0.f;
            for (int e = 0; e < D; ++e)
                dot = fmaf(__uint_as_float((uint32_t)qr[e] << 16), __uint_as_float((uint32_t)kb[(int64_t)j * D + e] << 16), dot);
            lse_merge(m, l, dot, 1.f, a.c);
        }
        if (l > 0.f) v = m + fast_log2(l) * a.inv_c;
    }
    out[(int64_t)phase * a.rows_pad + row] = v;
}

// ---------------------------------------------------------------------------
// prob: per key, sum over lookahead rows (and layers) of the head-maximum of
// the attention probability.
// ---------------------------------------------------------------------------
template <int D, int NS, int NB, bool FP8>
__global__ __launch_bounds__(kThreads, 3) void sp_prob_kernel(ScoreArgs a, LayerPtrs kp)
{
    constexpr int KS = D / 16;
    constexpr int TILE = kWaves * NS * 32;
    extern __shared__ u32x4 lds[];
    u32x4 *ks = lds;
    u32x4 *qs = lds + TILE * (D / 8);
    float *ci = reinterpret_cast<float *>(qs + a.rows_pad * (D / 8));   // rows_pad floats
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, hf = lane >> 5, col = lane & 31;
    const int tile = blockIdx.x, split = blockIdx.y;
    const TileInfo ti = get_tile(a, tile, TILE);
    const int n_phases = a.n_layers * a.n_kv_heads;
    const float c = a.c;
    const int layer_lo = split * a.layers_per_split;
    const int layer_hi = min(layer_lo + a.layers_per_split, a.n_layers);
    const bool whole = a.n_splits == 1;

    float mx[NS][NB][4];
    float total[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        total[s] = 0.f;
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int e = 0; e < 4; ++e) mx[s][b][e] = neg_inf();
    }

    for (int layer = layer_lo; layer < layer_hi; ++layer) {
        for (int kv = 0; kv < a.n_kv_heads; ++kv) {
            const int phase = layer * a.n_kv_heads + kv;
            __syncthreads();
            stage_q<D>(qs, a, ti.prompt, layer, kv, tid);
            if (FP8) stage_k_fp8<D, NS>(ks, key_base_fp8(a, kp, layer, kv), a.k_stride_token, ti.j0, ti.end, tid);
            else stage_k<D, NS>(ks, key_base(a, kp, layer, kv, ti), a.k_stride_token, ti.j0, ti.end, tid);
            // 8-bit keys: logit differences of this (layer, kv head) are in units of its stored keys; its scale
            // brings them to the common unit before they meet those of other heads and layers
            const float ksc = FP8 ? a.kscale[phase] : 1.0f;
            for (int i = tid; i < a.rows_pad; i += kThreads)
                ci[i] = a.lse_neg[((int64_t)ti.prompt * n_phases + phase) * a.rows_pad + i];
            __syncthreads();

            bf16x8 kf[NS][KS];
#pragma unroll
            for (int s = 0; s < NS; ++s) load_frag<D>(ks, (wave * NS + s) * 32 + col, hf, kf[s]);

#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                for (int gb = 0; gb < a.n_gblk; ++gb) {
                    const int blk = gb * NB + nb;
                    bf16x8 qf[KS];
                    load_frag<D>(qs, blk * 32 + col, hf, qf);
                    f32x16 cinit;
                    const float4 *cp = reinterpret_cast<const float4 *>(ci + blk * 32 + hf * 16);
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float4 x = cp[v];
                        cinit[4 * v + 0] = x.x; cinit[4 * v + 1] = x.y;
                        cinit[4 * v + 2] = x.z; cinit[4 * v + 3] = x.w;
                    }
#pragma unroll
                    for (int s = 0; s < NS; ++s) {
                        f32x16 acc = cinit;
#pragma unroll
                        for (int t = 0; t < KS; ++t)
                            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[t], kf[s][t], acc, 0, 0, 0);
                        // acc[r]: group head r/4, lookahead row 8*nb + 4*hf + r%4, key (wave*NS+s)*32 + col
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float v = fmaxf(fmaxf(acc[e], acc[4 + e]), fmaxf(acc[8 + e], acc[12 + e]));
                            mx[s][nb][e] = fmaxf(mx[s][nb][e], FP8 ? v * ksc : v);
                        }
                    }
                }
            }
        }
        if (a.layer_agg == SP_LAYER_MEAN || (whole && layer == a.n_layers - 1)) {
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                float sum = 0.f;
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        sum += fast_exp2(mx[s][b][e] * c);
                        mx[s][b][e] = neg_inf();
                    }
                total[s] += sum;
            }
        }
    }
    if (!whole && a.layer_agg == SP_LAYER_MAX) {
        // probabilities of this layer range's head-and-layer maxima, one per (lookahead row, key);
        // exp is monotone, so the maximum over ranges can be taken after it
        const int n_rows = 8 * NB;
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int n = 8 * b + 4 * hf + e;
                    a.split_buf[(((int64_t)split * n_rows + n) * a.n_tiles + tile) * TILE + (wave * NS + s) * 32 + col] =
                        fast_exp2(mx[s][b][e] * c);
                }
        return;
    }
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const float both = total[s] + __shfl_xor(total[s], 32);
        const int local = (wave * NS + s) * 32 + col;
        const int64_t j = ti.j0 + local;
        if (hf != 0) continue;
        if (!whole) a.split_buf[((int64_t)split * a.n_tiles + tile) * TILE + local] = both;
        else if (j < ti.end) a.scores[j] = both * a.out_scale;
    }
}

// ---------------------------------------------------------------------------
// reduce: combines the layer ranges of a split prob pass, one thread per key,
// ranges in ascending order. MEAN adds the ranges' sums; MAX takes, per
// lookahead row, the largest probability over the ranges and adds the rows.
// ---------------------------------------------------------------------------
template <int TILE>
__global__ __launch_bounds__(TILE) void sp_prob_reduce_kernel(ScoreArgs a)
{
    const int tile = blockIdx.x, local = threadIdx.x;
    const TileInfo ti = get_tile(a, tile, TILE);
    const int64_t j = ti.j0 + local;
    if (j >= ti.end) return;
    float sum = 0.f;
    if (a.layer_agg == SP_LAYER_MEAN) {
        for (int s = 0; s < a.n_splits; ++s) sum += a.split_buf[((int64_t)s * a.n_tiles + tile) * TILE + local];
    } else {
        const int n_rows = 8 * a.n_nblk;
        for (int n = 0; n < n_rows; ++n) {
            float m = 0.f;
            for (int s = 0; s < a.n_splits; ++s)
                m = fmaxf(m, a.split_buf[(((int64_t)s * n_rows + n) * a.n_tiles + tile) * TILE + local]);
            sum += m;
        }
    }
    a.scores[j] = sum * a.out_scale;
}

// Tile table of a ragged batch: tiles never straddle prompts.
__global__ void sp_tiles_kernel(const int64_t *offsets, int n_prompts, int tile_keys, TileInfo *tiles,
                                int32_t *prompt_tiles, int n_tiles_cap)
{
    for (int b = threadIdx.x; b <= n_prompts; b += blockDim.x) {
        int64_t first = 0;
        for (int p = 0; p < b; ++p) first += (offsets[p + 1] - offsets[p] + tile_keys - 1) / tile_keys;
        prompt_tiles[b] = (int32_t)first;
        if (b == n_prompts) continue;
        const int64_t beg = offsets[b], end = offsets[b + 1];
        int64_t t = first;
        for (int64_t j = beg; j < end && t < n_tiles_cap; j += tile_keys, ++t) {
            TileInfo ti;
            ti.j0 = j; ti.end = end; ti.prompt = b; ti.first_tile = (int32_t)first;
            tiles[t] = ti;
        }
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
struct Plan {
    int D, NS, NB, n_gblk, rows_pad, tile_keys, n_phases, n_layers, layer_agg;
    size_t lds_bytes;
};

// Layers per workgroup of the prob pass: all of them once the tiles alone fill the device.
int prob_layers_per_split(const Plan &p, int64_t n_tiles)
{
    int64_t want = (kProbTargetWgs + n_tiles - 1) / n_tiles;
    if (want < 1) want = 1;
    if (want > p.n_layers) want = p.n_layers;
    return (int)((p.n_layers + want - 1) / want);
}

int prob_splits(const Plan &p, int64_t n_tiles)
{
    const int lps = prob_layers_per_split(p, n_tiles);
    return (p.n_layers + lps - 1) / lps;
}

// Floats of the layer-split buffer, bounded over every tile count up to n_tiles (the workspace query
// rounds the tile count up): splits * tiles never exceeds either term of the minimum.
size_t split_buf_floats(const Plan &p, int64_t n_tiles)
{
    int64_t blocks = (int64_t)p.n_layers * n_tiles;
    if (blocks > kProbTargetWgs + n_tiles) blocks = kProbTargetWgs + n_tiles;
    const int per_key = (p.layer_agg == SP_LAYER_MAX) ? 8 * p.NB : 1;
    return (size_t)blocks * p.tile_keys * per_key;
}

sp_status make_plan(const sp_score_desc *d, Plan &p)
{
    if (!d) return sp::fail(SP_ERR_INVALID_ARG, "desc is null");
    if (d->n_layers < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->n_q < 1 || d->head_dim < 1)
        return sp::fail(SP_ERR_INVALID_ARG, "desc: sizes must be positive");
    if (d->n_q_heads % d->n_kv_heads != 0)
        return sp::fail(SP_ERR_INVALID_ARG, "desc: n_q_heads (%d) is not a multiple of n_kv_heads (%d)",
                        d->n_q_heads, d->n_kv_heads);
    if (!(d->scale > 0.f) || !std::isfinite(d->scale))
        return sp::fail(SP_ERR_INVALID_ARG, "desc: scale must be finite and > 0");
    if (d->layer_agg != SP_LAYER_MEAN && d->layer_agg != SP_LAYER_MAX)
        return sp::fail(SP_ERR_INVALID_ARG, "desc: layer_agg must be SP_LAYER_MEAN or SP_LAYER_MAX");
    if (d->head_dim != 64 && d->head_dim != 128)
        return sp::fail(SP_ERR_UNSUPPORTED, "desc: head_dim %d (supported: 64, 128)", d->head_dim);
    if (d->n_q > 16) return sp::fail(SP_ERR_UNSUPPORTED, "desc: n_q %d (supported: 1..16)", d->n_q);
    if (d->n_layers > kMaxLayers)
        return sp::fail(SP_ERR_UNSUPPORTED, "desc: n_layers %d (supported: <= %d)", d->n_layers, kMaxLayers);
    const int G = d->n_q_heads / d->n_kv_heads;
    if (G > 16) return sp::fail(SP_ERR_UNSUPPORTED, "desc: %d query heads per kv head (supported: <= 16)", G);
    if (d->k_stride_token < d->head_dim || d->k_stride_head < 0 || d->k_stride_token % 8 != 0 ||
        d->k_stride_head % 8 != 0)
        return sp::fail(SP_ERR_INVALID_ARG, "desc: K strides must be multiples of 8 elements, token stride >= head_dim");
    p.D = d->head_dim;
    p.NS = (p.D == 64) ? 2 : 1;
    p.NB = (d->n_q + 7) / 8;
    p.n_gblk = (G + 3) / 4;
    p.rows_pad = p.NB * p.n_gblk * 32;
    p.tile_keys = kWaves * p.NS * 32;
    p.n_phases = d->n_layers * d->n_kv_heads;
    if (p.n_phases > 65535)
        return sp::fail(SP_ERR_UNSUPPORTED, "desc: %d (layer, kv head) pairs (supported: <= 65535)", p.n_phases);
    p.n_layers = d->n_layers;
    p.layer_agg = d->layer_agg;
    p.lds_bytes = (size_t)p.tile_keys * p.D * 2 + (size_t)p.rows_pad * p.D * 2 + (size_t)p.rows_pad * 4;
    if (p.lds_bytes > kLdsBudget)
        return sp::fail(SP_ERR_UNSUPPORTED, "desc: query group of %d heads x %d rows at head_dim %d exceeds on-chip staging",
                        G, d->n_q, p.D);
    return SP_OK;
}

struct WsLayout {
    size_t status, part, lse, tiles, prompt_tiles, split, look, fused, total;
};

// Shapes the fused single-launch kernel can hold on chip (any L; the length test is separate).
bool fused_shape_ok(const Plan &p)
{
    return p.D == 64 ? p.rows_pad <= sp_fused::kMaxRows : p.rows_pad <= sp_fused::kMaxRowsWide;
}

// Keys a workgroup of the fused kernel owns: 512 at head_dim 64, 256 at head_dim 128 (twice the tile of
// the two-pass path), and the fewest workgroups it is used with.
int fused_tile(const Plan &p) { return p.D == 64 ? sp_fused::kTileKeys : sp_fused::kTileKeys / 2; }
int fused_min_workgroups(const Plan &p) { return p.D == 64 ? sp_fused::kMinWorkgroups : sp_fused::kMinWorkgroupsWide; }

int fused_workgroups(const Plan &p, int64_t L)
{
    const int64_t n = sp::ceil_div(L, fused_tile(p));
    return n > 0x7fffffff ? 0x7fffffff : (int)n;
}

bool fused_applies(const Plan &p, int64_t L, int64_t k_stride_token);

// Compute units of the current device (0 if it cannot be queried); the fused kernel needs one per workgroup.
int device_compute_units()
{
    static thread_local int cached_dev = -1, cached_cus = 0;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (dev != cached_dev) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 0;
        if (cus > 0 && !sp_fused::fits_one_per_cu()) cus = 0;
        cached_dev = dev;
        cached_cus = cus;
    }
    return cached_cus;
}

// The fused kernel runs one workgroup of 512 keys per compute unit: long single prompts only.
bool fused_applies(const Plan &p, int64_t L, int64_t k_stride_token)
{
    if (!fused_shape_ok(p)) return false;
    if (k_stride_token > (int64_t(1) << 20)) return false;       // lane offsets within a tile are 32-bit
    const int n_wg = fused_workgroups(p, L);
    return n_wg >= fused_min_workgroups(p) && n_wg <= 256 && n_wg <= device_compute_units();
}

// 8-bit keys: the single-launch kernel's variants for them fetch the codes in 16-byte pieces (strides in
// multiples of 16 elements).
bool fused_applies_fp8(const Plan &p, const sp_score_desc *desc, int64_t L)
{
    return desc->k_stride_token % 16 == 0 && desc->k_stride_head % 16 == 0 && fused_applies(p, L, desc->k_stride_token);
}

// A ragged batch on the single-launch kernel: the prompts are packed into launches of at most one
// workgroup per compute unit (first fit, longest first), each prompt with all its 512-key tiles in one
// launch. Applies when every prompt is empty or at least one tile long and fits a launch, the batch has
// enough tiles to be worth it, and every launch has at least as many workgroups as duty blocks.
struct BatchGroups {
    std::vector<sp_fused::GroupTable> groups;
    std::vector<int> wgs;
};

bool plan_fused_batch(const Plan &p, const int64_t *offsets, int B, int64_t k_stride_token, BatchGroups &out)
{
    if (!fused_shape_ok(p) || k_stride_token > (int64_t(1) << 20)) return false;
    const int cap = std::min(256, device_compute_units());
    if (cap < sp_fused::kMinWorkgroups) return false;
    std::vector<std::pair<int, int>> order;        // (tiles, prompt)
    int64_t total_tiles = 0;
    for (int b = 0; b < B; ++b) {
        const int64_t len = offsets[b + 1] - offsets[b];
        if (len == 0) continue;
        if (len < fused_tile(p)) return false;
        const int64_t tiles = sp::ceil_div(len, fused_tile(p));
        if (tiles > cap) return false;
        order.emplace_back((int)tiles, b);
        total_tiles += tiles;
    }
    if (total_tiles < sp_fused::kMinWorkgroups) return false;
    std::stable_sort(order.begin(), order.end(), [](const std::pair<int, int> &x, const std::pair<int, int> &y) { return x.first > y.first; });
    out.groups.clear();
    out.wgs.clear();
    for (const auto &tp : order) {
        size_t g = 0;
        for (; g < out.groups.size(); ++g)
            if (out.wgs[g] + tp.first <= cap && out.groups[g].n < sp_fused::kMaxGroupPrompts) break;
        if (g == out.groups.size()) {
            sp_fused::GroupTable t;
            std::memset(&t, 0, sizeof t);
            out.groups.push_back(t);
            out.wgs.push_back(0);
        }
        sp_fused::GroupTable &t = out.groups[g];
        t.prompt[t.n] = tp.second;
        t.start[t.n] = offsets[tp.second];
        t.len[t.n] = offsets[tp.second + 1] - offsets[tp.second];
        t.w0[t.n] = out.wgs[g];
        out.wgs[g] += tp.first;
        t.w0[++t.n] = out.wgs[g];
    }
    for (size_t g = 0; g < out.groups.size(); ++g)
        if (out.groups[g].n * (p.rows_pad / 4) > out.wgs[g]) return false;      // more duty blocks than workgroups
    return true;
}

WsLayout ws_layout(const Plan &p, int64_t n_tiles, int n_prompts)
{
    WsLayout w;
    size_t off = 0;
    w.status = off; off += 256;           // the call's status word leads the workspace (see sp.h)
    w.part = off;  off = sp::align_up(off + sizeof(float2) * (size_t)p.n_phases * (size_t)n_tiles * p.rows_pad, 256);
    w.lse = off;   off = sp::align_up(off + sizeof(float) * (size_t)n_prompts * p.n_phases * p.rows_pad, 256);
    w.tiles = off; off = sp::align_up(off + sizeof(TileInfo) * (size_t)n_tiles, 256);
    w.prompt_tiles = off; off = sp::align_up(off + sizeof(int32_t) * (size_t)(n_prompts + 1), 256);
    w.split = off; off = sp::align_up(off + sizeof(float) * split_buf_floats(p, n_tiles), 256);
    w.look = off; off = sp::align_up(off + sizeof(float) * (size_t)p.n_phases * p.rows_pad, 256);
    w.fused = off;
    if (fused_shape_ok(p)) {
        int64_t n_wg = n_tiles * p.tile_keys / fused_tile(p) + n_prompts;
        if (n_wg > 1024) n_wg = 1024;
        off += sp_fused::workspace_bytes(p.rows_pad, (int)n_wg, std::min(n_prompts, sp_fused::kMaxGroupPrompts));
    }
    w.total = off;
    return w;
}

template <int D, int NS, bool FP8 = false>
sp_status launch_all(const Plan &p, const ScoreArgs &a, const LayerPtrs &kp, hipStream_t st)
{
    const dim3 block(kThreads);
    hipLaunchKernelGGL((sp_stats_kernel<D, NS, FP8>), dim3(a.n_tiles, p.n_phases), block, p.lds_bytes, st, a, kp);
    SP_HIP_CHECK(hipGetLastError());
    hipLaunchKernelGGL(sp_merge_kernel, dim3(p.rows_pad / 32, p.n_phases, a.n_prompts), dim3(kMergeThreads), 0, st, a);
    SP_HIP_CHECK(hipGetLastError());
    const dim3 grid(a.n_tiles, a.n_splits);
    if (p.NB == 1)
        hipLaunchKernelGGL((sp_prob_kernel<D, NS, 1, FP8>), grid, block, p.lds_bytes, st, a, kp);
    else
        hipLaunchKernelGGL((sp_prob_kernel<D, NS, 2, FP8>), grid, block, p.lds_bytes, st, a, kp);
    SP_HIP_CHECK(hipGetLastError());
    if (a.n_splits > 1) {
        constexpr int TILE = kWaves * NS * 32;
        hipLaunchKernelGGL((sp_prob_reduce_kernel<TILE>), dim3(a.n_tiles), dim3(TILE), 0, st, a);
        SP_HIP_CHECK(hipGetLastError());
    }
    return SP_OK;
}

// What the variants of sp_score add to the plain call.
struct ScoreOptions {
    const void *k_look = nullptr;            // lookahead keys in the normaliser
    int32_t look_self = 0;
    const int32_t *block_table = nullptr;    // paged keys
    int64_t page_tokens = 0, page_stride = 0;
    const float *kscale = nullptr;           // 8-bit keys with these scales
};

sp_status score_impl(const sp_score_desc *desc, const void *q_dev, const void *const *k_layers_host,
                     const int64_t *offsets_host, const int64_t *offsets_dev, int32_t B, int64_t L_single,
                     const ScoreOptions &opt, float *scores_dev, void *ws_dev, size_t ws_bytes, void *hip_stream)
{
    Plan p;
    sp_status rc = make_plan(desc, p);
    if (rc != SP_OK) return rc;
    if (!q_dev || !k_layers_host || !scores_dev)
        return sp::fail(SP_ERR_INVALID_ARG, "q_dev, k_layers_host and scores_dev must not be null");
    LayerPtrs kp;
    std::memset(&kp, 0, sizeof kp);
    for (int l = 0; l < desc->n_layers; ++l) {
        if (!k_layers_host[l]) return sp::fail(SP_ERR_INVALID_ARG, "k_layers_host[%d] is null", l);
        if ((uintptr_t)k_layers_host[l] % 16 != 0)
            return sp::fail(SP_ERR_INVALID_ARG, "k_layers_host[%d] is not 16-byte aligned", l);
        kp.p[l] = static_cast<const uint16_t *>(k_layers_host[l]);
    }
    if ((uintptr_t)q_dev % 16 != 0) return sp::fail(SP_ERR_INVALID_ARG, "q_dev is not 16-byte aligned");
    if (opt.look_self != 0 && opt.look_self != 1)
        return sp::fail(SP_ERR_INVALID_ARG, "look_self = %d must be 0 or 1", opt.look_self);
    if (opt.block_table) {
        // a page holds whole tiles of either score path, and its rows are addressed with the desc's strides
        if (opt.page_tokens < sp_fused::kTileKeys || opt.page_tokens % sp_fused::kTileKeys != 0)
            return sp::fail(SP_ERR_INVALID_ARG, "page_tokens = %lld must be a positive multiple of %d",
                            (long long)opt.page_tokens, sp_fused::kTileKeys);
        if (opt.page_stride < 0 || opt.page_stride % 8 != 0)
            return sp::fail(SP_ERR_INVALID_ARG, "page_stride = %lld must be a non-negative multiple of 8 elements",
                            (long long)opt.page_stride);
    }

    int64_t total = 0, n_tiles = 0;
    const bool batch = offsets_host != nullptr;
    if (batch) {
        if (!offsets_dev) return sp::fail(SP_ERR_INVALID_ARG, "offsets_dev is null");
        if (B < 1 || B > kMaxPrompts) return sp::fail(SP_ERR_INVALID_ARG, "B = %d (supported: 1..%d)", B, kMaxPrompts);
        if (offsets_host[0] != 0) return sp::fail(SP_ERR_INVALID_ARG, "offsets_host[0] must be 0");
        for (int b = 0; b < B; ++b) {
            const int64_t len = offsets_host[b + 1] - offsets_host[b];
            if (len < 0) return sp::fail(SP_ERR_INVALID_ARG, "offsets_host decreases at prompt %d", b);
            n_tiles += sp::ceil_div(len, p.tile_keys);
        }
        total = offsets_host[B];
    } else {
        if (L_single < 0) return sp::fail(SP_ERR_INVALID_ARG, "L = %lld is negative", (long long)L_single);
        total = L_single;
        n_tiles = sp::ceil_div(total, p.tile_keys);
        B = 1;
    }
    if (total == 0) return SP_OK;
    if (n_tiles > 0x7fffffff / 2) return sp::fail(SP_ERR_UNSUPPORTED, "too many key tiles (%lld)", (long long)n_tiles);

    const WsLayout w = ws_layout(p, n_tiles, B);
    if (!ws_dev) return sp::fail(SP_ERR_WORKSPACE, "ws_dev is null (%zu bytes needed)", w.total);
    if ((uintptr_t)ws_dev % 256 != 0) return sp::fail(SP_ERR_WORKSPACE, "ws_dev is not 256-byte aligned");
    if (ws_bytes < w.total) return sp::fail(SP_ERR_WORKSPACE, "workspace too small: %zu < %zu", ws_bytes, w.total);

    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char *ws = static_cast<char *>(ws_dev);
    ScoreArgs a;
    std::memset(&a, 0, sizeof a);
    a.q = static_cast<const uint16_t *>(q_dev);
    a.k_stride_token = desc->k_stride_token;
    a.k_stride_head = desc->k_stride_head;
    a.L = total;
    a.part = reinterpret_cast<float2 *>(ws + w.part);
    a.lse_neg = reinterpret_cast<float *>(ws + w.lse);
    a.scores = scores_dev;
    a.status = reinterpret_cast<uint32_t *>(ws + w.status);
    a.split_buf = reinterpret_cast<float *>(ws + w.split);
    a.layers_per_split = prob_layers_per_split(p, n_tiles);
    a.n_splits = prob_splits(p, n_tiles);
    a.n_tiles = (int32_t)n_tiles;
    a.n_prompts = B;
    a.n_layers = desc->n_layers;
    a.n_q_heads = desc->n_q_heads;
    a.n_kv_heads = desc->n_kv_heads;
    a.group = desc->n_q_heads / desc->n_kv_heads;
    a.n_q = desc->n_q;
    a.n_nblk = p.NB;
    a.n_gblk = p.n_gblk;
    a.rows_pad = p.rows_pad;
    a.layer_agg = desc->layer_agg;
    a.c = desc->scale * 1.44269504088896340736f;
    a.inv_c = 1.0f / a.c;
    a.out_scale = (desc->layer_agg == SP_LAYER_MAX) ? 1.0f / (float)desc->n_q
                                                   : 1.0f / ((float)desc->n_q * (float)desc->n_layers);
    a.block_table = opt.block_table;
    a.page_tokens = opt.page_tokens;
    a.page_stride = opt.page_stride;
    a.kscale = opt.kscale;
    if (opt.k_look) {
        float *look = reinterpret_cast<float *>(ws + w.look);
        hipLaunchKernelGGL(sp_look_kernel, dim3(p.n_phases), dim3(kThreads), 0, st, a,
                           static_cast<const uint16_t *>(opt.k_look), (int)opt.look_self, p.D, look);
        SP_HIP_CHECK(hipGetLastError());
        a.look = look;
    }
    // 8-bit keys outside the single-launch kernel's variant for them take the three-kernel path
    const bool fp8_fused = opt.kscale && !batch && fused_applies_fp8(p, desc, total);
    if (opt.kscale && !fp8_fused) {
        if (p.D == 64) return launch_all<64, 2, true>(p, a, kp, st);
        return launch_all<128, 1, true>(p, a, kp, st);
    }
    if (!batch && fused_applies(p, total, desc->k_stride_token)) {
        const int n_wg = fused_workgroups(p, total);
        {
            sp_fused::FusedArgs f;
            std::memset(&f, 0, sizeof f);
            f.q = a.q;
            f.head_dim = p.D;
            f.tile_keys = fused_tile(p);
            f.k_stride_token = a.k_stride_token;
            f.k_stride_head = a.k_stride_head;
            f.L = total;
            f.kscale = opt.kscale;
            f.look = a.look;
            f.block_table = a.block_table;
            f.page_tokens = a.page_tokens;
            f.page_stride = a.page_stride;
            f.scores = scores_dev;
            f.n_wg = n_wg;
            f.n_layers = a.n_layers; f.n_q_heads = a.n_q_heads; f.n_kv_heads = a.n_kv_heads;
            f.group = a.group; f.n_q = a.n_q;
            f.n_nblk = a.n_nblk; f.n_gblk = a.n_gblk; f.rows_pad = a.rows_pad;
            f.layer_agg = a.layer_agg;
            f.c = a.c; f.inv_c = a.inv_c; f.out_scale = a.out_scale;
            return sp_fused::launch(f, kp, nullptr, true, ws + w.fused, a.status, st);
        }
    }
    BatchGroups bg;
    if (batch && !opt.k_look && !opt.block_table && plan_fused_batch(p, offsets_host, B, desc->k_stride_token, bg)) {
        for (size_t g = 0; g < bg.groups.size(); ++g) {
            sp_fused::FusedArgs f;
            std::memset(&f, 0, sizeof f);
            f.q = a.q;
            f.head_dim = p.D;
            f.tile_keys = fused_tile(p);
            f.k_stride_token = a.k_stride_token;
            f.k_stride_head = a.k_stride_head;
            f.L = 0;
            f.scores = scores_dev;
            f.n_wg = bg.wgs[g];
            f.n_layers = a.n_layers; f.n_q_heads = a.n_q_heads; f.n_kv_heads = a.n_kv_heads;
            f.group = a.group; f.n_q = a.n_q;
            f.n_nblk = a.n_nblk; f.n_gblk = a.n_gblk; f.rows_pad = a.rows_pad;
            f.layer_agg = a.layer_agg;
            f.c = a.c; f.inv_c = a.inv_c; f.out_scale = a.out_scale;
            const sp_status rs = sp_fused::launch(f, kp, &bg.groups[g], g == 0, ws + w.fused, a.status, st);
            if (rs != SP_OK) return rs;
        }
        return SP_OK;
    }
    if (batch) {
        TileInfo *tiles = reinterpret_cast<TileInfo *>(ws + w.tiles);
        int32_t *pt = reinterpret_cast<int32_t *>(ws + w.prompt_tiles);
        hipLaunchKernelGGL(sp_tiles_kernel, dim3(1), dim3(256), 0, st, offsets_dev, B, p.tile_keys, tiles, pt,
                           (int)n_tiles);
        SP_HIP_CHECK(hipGetLastError());
        a.tiles = tiles;
        a.prompt_tiles = pt;
    }
    if (p.D == 64) return launch_all<64, 2>(p, a, kp, st);
    return launch_all<128, 1>(p, a, kp, st);
}

}  // namespace

extern "C" sp_status sp_score_workspace(const sp_score_desc *desc, int64_t total_tokens, int32_t n_prompts,
                                        size_t *bytes)
{
    Plan p;
    sp_status rc = make_plan(desc, p);
    if (rc != SP_OK) return rc;
    if (!bytes) return sp::fail(SP_ERR_INVALID_ARG, "bytes is null");
    if (total_tokens < 0 || n_prompts < 1 || n_prompts > kMaxPrompts)
        return sp::fail(SP_ERR_INVALID_ARG, "total_tokens must be >= 0 and n_prompts in 1..%d", kMaxPrompts);
    const int64_t n_tiles = sp::ceil_div(total_tokens, p.tile_keys) + n_prompts;
    *bytes = ws_layout(p, n_tiles, n_prompts).total;
    return SP_OK;
}

extern "C" void sp_debug_fused_giveup(uint32_t spin_limit, int32_t force_miss)
{
    sp_fused::set_giveup(spin_limit, force_miss);
}

extern "C" int32_t sp_score_is_fused(const sp_score_desc *desc, int64_t L)
{
    Plan p;
    if (make_plan(desc, p) != SP_OK) return -1;
    return fused_applies(p, L, desc->k_stride_token) ? 1 : 0;
}

extern "C" int32_t sp_score_fp8_is_fused(const sp_score_desc *desc, int64_t L)
{
    Plan p;
    if (make_plan(desc, p) != SP_OK) return -1;
    return fused_applies_fp8(p, desc, L) ? 1 : 0;
}

extern "C" int32_t sp_score_batch_is_fused(const sp_score_desc *desc, const int64_t *offsets_host, int32_t B)
{
    Plan p;
    if (make_plan(desc, p) != SP_OK || !offsets_host || B < 1 || B > kMaxPrompts) return -1;
    for (int b = 0; b < B; ++b)
        if (offsets_host[b + 1] < offsets_host[b]) return -1;
    BatchGroups bg;
    return plan_fused_batch(p, offsets_host, B, desc->k_stride_token, bg) ? (int32_t)bg.groups.size() : 0;
}

extern "C" sp_status sp_score(const sp_score_desc *desc, const void *q_dev, const void *const *k_layers_host,
                              int64_t L, float *scores_dev, void *ws_dev, size_t ws_bytes, void *hip_stream)
{
    return score_impl(desc, q_dev, k_layers_host, nullptr, nullptr, 1, L, ScoreOptions(), scores_dev, ws_dev, ws_bytes,
                      hip_stream);
}

extern "C" sp_status sp_score_look(const sp_score_desc *desc, const void *q_dev, const void *const *k_layers_host,
                                   int64_t L, const void *k_look_dev, int32_t look_self, float *scores_dev,
                                   void *ws_dev, size_t ws_bytes, void *hip_stream)
{
    if (!k_look_dev) return sp::fail(SP_ERR_INVALID_ARG, "k_look_dev is null");
    if ((uintptr_t)k_look_dev % 16 != 0) return sp::fail(SP_ERR_INVALID_ARG, "k_look_dev is not 16-byte aligned");
    ScoreOptions opt;
    opt.k_look = k_look_dev;
    opt.look_self = look_self;
    return score_impl(desc, q_dev, k_layers_host, nullptr, nullptr, 1, L, opt, scores_dev, ws_dev, ws_bytes, hip_stream);
}

extern "C" sp_status sp_score_paged(const sp_score_desc *desc, const void *q_dev, const void *const *k_pools_host,
                                    const int32_t *block_table_dev, int64_t page_tokens, int64_t page_stride, int64_t L,
                                    float *scores_dev, void *ws_dev, size_t ws_bytes, void *hip_stream)
{
    if (!block_table_dev) return sp::fail(SP_ERR_INVALID_ARG, "block_table_dev is null");
    ScoreOptions opt;
    opt.block_table = block_table_dev;
    opt.page_tokens = page_tokens;
    opt.page_stride = page_stride;
    return score_impl(desc, q_dev, k_pools_host, nullptr, nullptr, 1, L, opt, scores_dev, ws_dev, ws_bytes, hip_stream);
}

extern "C" sp_status sp_score_fp8(const sp_score_desc *desc, const void *q_dev, const void *const *k8_layers_host,
                                  const float *kscale_dev, int64_t L, float *scores_dev, void *ws_dev, size_t ws_bytes,
                                  void *hip_stream)
{
    if (!kscale_dev) return sp::fail(SP_ERR_INVALID_ARG, "kscale_dev is null");
    ScoreOptions opt;
    opt.kscale = kscale_dev;
    return score_impl(desc, q_dev, k8_layers_host, nullptr, nullptr, 1, L, opt, scores_dev, ws_dev, ws_bytes, hip_stream);
}

extern "C" sp_status sp_score_batch(const sp_score_desc *desc, const void *q_dev, const void *const *k_layers_host,
                                    const int64_t *offsets_host, const int64_t *offsets_dev, int32_t B,
                                    float *scores_dev, void *ws_dev, size_t ws_bytes, void *hip_stream)
{
    if (!offsets_host) return sp::fail(SP_ERR_INVALID_ARG, "offsets_host is null");
    return score_impl(desc, q_dev, k_layers_host, offsets_host, offsets_dev, B, 0, ScoreOptions(), scores_dev, ws_dev,
                      ws_bytes, hip_stream);
}

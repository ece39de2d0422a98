// Fused single-launch sp_score for long prompts: every K row is read from HBM
// exactly once (paper: Appendix A.1.1; Algorithm 1 "AggregateMaxMean").
//
// The exact softmax needs each row's normaliser (a reduction over all L keys)
// before any probability can be formed, and the head maximum must be taken on
// normalised values. Reading K a second time would halve the achievable rate,
// so this kernel keeps K on chip between the two uses:
//
//  * one persistent workgroup per compute unit (8 waves) owns 512 consecutive
//    keys for the whole call; a "phase" is one (layer, kv head) pair, and the
//    workgroup's share of a phase is a 512 x 64 bf16 tile (64 KB);
//  * tiles stream HBM -> LDS with direct-to-LDS loads, two phases ahead, into
//    two transit buffers; each wave lifts its 64 keys into MFMA fragments held
//    in registers (a ring of three phases);
//  * phase p: the statistics pass computes the partial (max, sum exp) of every
//    query row over the workgroup's keys and publishes it to global memory;
//  * one wave of some workgroup (rotating "duty") combines the partials of one
//    row over all workgroups in a fixed order and publishes the normaliser;
//  * three phases later the workgroup picks the normalisers up and runs the
//    probability pass of phase p from the fragments still in its registers:
//    logits again with -lse folded into the MFMA accumulator, maximum over
//    heads on logits, one exp per (lookahead row, key), accumulation over
//    lookahead rows and layers in registers. Scores are stored once at the end.
//
// The exchange uses no read-modify-write atomics and no cache-wide fences:
// every exchanged word is written and read with device-scope relaxed atomics,
// readiness travels inside the data (the sign bit of the always-positive sum
// carries the parity of the slot's use; normalisers carry the phase number),
// and all waits are bounded. The grid never exceeds the number of compute units
// (one workgroup fits per unit), so every workgroup is resident on an idle device.
#include "sp_score_fused.hpp"

#include <cstring>

namespace {

using namespace sp_dev;
using sp_fused::FusedArgs;

constexpr int kD = 64;
constexpr int kCH = kD / 8;               // 16-byte chunks per key row
constexpr int kKS = kD / 16;              // MFMA k-steps per row
constexpr int kFWaves = 8;
constexpr int kFThreads = kFWaves * 64;
constexpr int kNS = 2;                    // 32-key sub-tiles per wave
constexpr int kFTile = sp_fused::kTileKeys;   // 512 keys per workgroup per phase
constexpr int kLag = 3;                   // phases between statistics and probability pass
constexpr int kSlots = sp_fused::kSlots;  // exchange ring depth
constexpr int kMaxRowsF = sp_fused::kMaxRows;   // 64 padded query rows per kv head
constexpr unsigned kSpinMax = 1u << 20;    // polls before a wait gives up (about a second)

#define SP_GPTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define SP_LPTR(p) ((__attribute__((address_space(3))) void *)(p))

__device__ __forceinline__ uint64_t ld64(const uint64_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st64(uint64_t *p, uint64_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Workgroup barrier that orders LDS traffic only. Direct-to-LDS loads are
// waited for explicitly (vm_wait) by the wave that issued them, so that younger
// loads can stay in flight across the barrier.
__device__ __forceinline__ void lds_barrier()
{
    __asm__ volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    __asm__ volatile("" ::: "memory");
}
// Wait until at most N vector-memory operations of this wave are outstanding.
template <int N>
__device__ __forceinline__ void vm_wait()
{
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
    __asm__ volatile("" ::: "memory");
}

struct Ring {
    bf16x8 kf[kLag][kNS][kKS];            // K fragments of the three phases in flight
};

struct PhaseId { int layer, kv; };
__device__ __forceinline__ PhaseId phase_of(int p, int n_kv) { PhaseId r; r.layer = p / n_kv; r.kv = p - r.layer * n_kv; return r; }

// padded query row -> (group head, lookahead row); see the row order in sp_score.hip
__device__ __forceinline__ bool row_valid(const FusedArgs &a, int row, int &g, int &n)
{
    const int blk = row >> 5, rho = row & 31;
    const int gblk = blk / a.n_nblk, nblk = blk - gblk * a.n_nblk;
    g = 4 * gblk + (rho >> 3);
    n = 8 * nblk + (rho & 7);
    return g < a.group && n < a.n_q;
}

// One wave instruction moves 64 chunks (8 key rows) of the tile; wave w issues
// instructions w, w+8, ... so the 8 waves cover the 512 rows.
__device__ __forceinline__ void issue_k_tile(u32x4 *kt, const uint16_t *slab, int64_t stride_token, int64_t j0,
                                             int n_valid, int wave, int lane)
{
    const int base_row = wave * 8 + (lane >> 3);
    const int chunk = (lane & 7) ^ ((base_row >> 1) & 7);     // (row >> 1) & 7 is the same for row + 64*i
#pragma unroll
    for (int i = 0; i < kFTile / 64; ++i) {
        int row = base_row + 64 * i;
        row = row < n_valid ? row : n_valid - 1;              // tail rows repeat the last valid key
        const uint16_t *src = slab + (j0 + row) * stride_token + chunk * 8;
        __builtin_amdgcn_global_load_lds(SP_GPTR(src), SP_LPTR(kt + (i * 8 + wave) * 64), 16, 0, 0);
    }
}

// Q tile of one (layer, kv head) in the padded row order. Every wave always issues exactly one
// instruction (8 rows); padding rows read a zero line kept in the workspace.
__device__ __forceinline__ void issue_q_tile(u32x4 *qt, const FusedArgs &a, int layer, int kv, int wave, int lane)
{
    const int row = wave * 8 + (lane >> 3);
    int g, n;
    const uint16_t *src = reinterpret_cast<const uint16_t *>(a.zeros) + (lane & 7) * 8;
    if (row < a.rows_pad && row_valid(a, row, g, n)) {
        const int chunk = (lane & 7) ^ ((row >> 1) & 7);
        src = a.q + ((((int64_t)layer * a.n_q_heads + (int64_t)kv * a.group + g) * a.n_q + n) * kD) + chunk * 8;
    }
    __builtin_amdgcn_global_load_lds(SP_GPTR(src), SP_LPTR(qt + wave * 64), 16, 0, 0);
}

template <int NB>
struct Acc {
    float mx[kNS][NB][4];
    float total[kNS];
};

// ---- probability pass of one phase from the fragment ring ----
template <int NB>
__device__ __forceinline__ void prob_pass(const FusedArgs &a, const bf16x8 (&kf)[kNS][kKS], const u32x4 *q2,
                                          const float *cinit, Acc<NB> &acc, int hf, int col)
{
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        for (int gb = 0; gb < a.n_gblk; ++gb) {
            const int blk = gb * NB + nb;
            bf16x8 qf[kKS];
            load_frag<kD>(q2, blk * 32 + col, hf, qf);
            f32x16 ci;
            const float4 *cp = reinterpret_cast<const float4 *>(cinit + blk * 32 + hf * 16);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float4 x = cp[v];
                ci[4 * v + 0] = x.x; ci[4 * v + 1] = x.y; ci[4 * v + 2] = x.z; ci[4 * v + 3] = x.w;
            }
#pragma unroll
            for (int s = 0; s < kNS; ++s) {
                f32x16 d = ci;
#pragma unroll
                for (int t = 0; t < kKS; ++t) d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[t], kf[s][t], d, 0, 0, 0);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float v = fmaxf(fmaxf(d[e], d[4 + e]), fmaxf(d[8 + e], d[12 + e]));
                    acc.mx[s][nb][e] = fmaxf(acc.mx[s][nb][e], v);
                }
            }
        }
    }
}

template <int NB>
__device__ __forceinline__ void close_layer(Acc<NB> &acc, float c)
{
#pragma unroll
    for (int s = 0; s < kNS; ++s) {
        float sum = 0.f;
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                sum += fast_exp2(acc.mx[s][b][e] * c);
                acc.mx[s][b][e] = neg_inf();
            }
        acc.total[s] += sum;
    }
}

// ---- statistics pass of one phase: per-wave (max, sum exp) of every row into wstats ----
__device__ __forceinline__ void stats_pass(const FusedArgs &a, const bf16x8 (&kf)[kNS][kKS], const u32x4 *q1,
                                           float2 *wstats_wave, int n_valid, int wave, int hf, int col)
{
    const float c = a.c;
    const int n_blk = a.rows_pad >> 5;
    for (int blk = 0; blk < n_blk; ++blk) {
        bf16x8 qf[kKS];
        load_frag<kD>(q1, blk * 32 + col, hf, qf);
        float m = neg_inf(), l = 0.f;
#pragma unroll
        for (int s = 0; s < kNS; ++s) {
            f32x16 d = {0.f};
#pragma unroll
            for (int t = 0; t < kKS; ++t) d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s][t], qf[t], d, 0, 0, 0);
            // d[r]: key (wave*2+s)*32 + 8*(r/4) + 4*hf + r%4 of the tile, query row blk*32 + col
            const int left = n_valid - (wave * kNS + s) * 32;
            if (left >= 32) {
                float tm = d[0];
#pragma unroll
                for (int r = 1; r < 16; ++r) tm = fmaxf(tm, d[r]);
                const float mn = fmaxf(m, tm);
                l *= fast_exp2((m - mn) * c);
                m = mn;
                const float mc = mn * c;
                float sum = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) sum += fast_exp2(fmaf(d[r], c, -mc));
                l += sum;
            } else if (left > 0) {
                float tm = neg_inf();
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = 8 * (r >> 2) + 4 * hf + (r & 3);
                    if (key < left) tm = fmaxf(tm, d[r]);
                }
                if (tm > neg_inf()) {
                    const float mn = fmaxf(m, tm);
                    l *= fast_exp2((m - mn) * c);
                    m = mn;
                    const float mc = mn * c;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = 8 * (r >> 2) + 4 * hf + (r & 3);
                        if (key < left) l += fast_exp2(fmaf(d[r], c, -mc));
                    }
                }
            }
        }
        const float m2 = __shfl_xor(m, 32), l2 = __shfl_xor(l, 32);
        lse_merge(m, l, m2, l2, c);
        if (hf == 0) wstats_wave[blk * 32 + col] = make_float2(m, l);
    }
}

struct Pending {
    uint64_t lse_entry;       // wave 0: normaliser entry of the phase whose probability pass comes next
    uint64_t duty[4];         // wave 1: partials of the duty row
};

// A partial is ready when it carries the parity of this use of its slot and a non-zero sum.
__device__ __forceinline__ bool duty_ready(const Pending &pend, uint32_t par)
{
    bool ok = true;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        ok = ok && ((uint32_t)(pend.duty[q] >> 63) == par) && ((pend.duty[q] >> 32) & 0x7fffffffu) != 0;
    return ok;
}

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// Row of phase p that workgroup w combines (>= rows_pad: none). Rows rotate over the workgroups.
__device__ __forceinline__ int duty_row_of(const FusedArgs &a, int p, int w)
{
    const int first = (int)(((int64_t)p * a.rows_pad) % a.n_wg);
    int r = w - first;
    return r < 0 ? r + a.n_wg : r;
}

// One iteration of the software pipeline. Every wave issues the same vector-memory instructions in
// the same order in every iteration (exchange loads of waves 0/1 aside), the eight K-tile loads last,
// so "at most eight outstanding" always means "everything but the newest K tile has landed".
template <int NB, int SLOT, int BUF>
__device__ __forceinline__ void iteration(const FusedArgs &a, const LayerPtrs &kp, int it, int n_phases, Ring &ring,
                                          Acc<NB> &acc, Pending &pend, u32x4 *kt0, u32x4 *kt1, u32x4 *q1, u32x4 *q2,
                                          float2 (*wstats)[kMaxRowsF], float *cinit, int *s_fail, int n_valid)
{
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, hf = lane >> 5, col = lane & 31;
    const int w = blockIdx.x;
    u32x4 *kt = BUF ? kt1 : kt0;
    const int pc = it - kLag;             // phase whose probability pass runs now
    const int pd = it - 2;                // phase whose duty loads were issued last iteration

    // ---- S1: take in what was requested last iteration ----
    vm_wait<kFTile / 64>();
    if (wave == 1 && pd >= 0 && pd < n_phases) {
        const int duty_row = duty_row_of(a, pd, w);
        int g, n;
        if (duty_row < a.rows_pad && row_valid(a, duty_row, g, n)) {
            const uint32_t par = (uint32_t)(pd / kSlots) & 1u;
            const uint64_t *src = a.part + ((size_t)(pd % kSlots) * a.rows_pad + duty_row) * a.n_wg;
            // fast path: the partials requested last iteration are all there; otherwise poll (bounded)
            if (__any(!duty_ready(pend, par)) && *s_fail == 0) {
                unsigned spins = 0;
                do {
                    if (++spins > kSpinMax) { *s_fail = 1; break; }
#pragma unroll
                    for (int q = 0; q < 4; ++q) pend.duty[q] = ld64(src + min(lane + 64 * q, a.n_wg - 1));
                } while (__any(!duty_ready(pend, par)));
            }
            float m = neg_inf(), l = 0.f;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float pm = __uint_as_float((uint32_t)pend.duty[q]);
                const float pl = __uint_as_float((uint32_t)(pend.duty[q] >> 32) & 0x7fffffffu);
                if (lane + 64 * q < a.n_wg) lse_merge(m, l, pm, pl, a.c);
            }
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const float m2 = __shfl_xor(m, off), l2 = __shfl_xor(l, off);
                lse_merge(m, l, m2, l2, a.c);
            }
            if (lane == 0) {
                const float v = -(m + fast_log2(l) * a.inv_c);
                st64(a.lse + (size_t)(pd % kSlots) * a.rows_pad + duty_row,
                     (uint64_t)__float_as_uint(v) | ((uint64_t)(uint32_t)(pd + 1) << 32));
            }
        }
    }
    if (wave == 0 && pc >= 0 && pc < n_phases && lane < a.rows_pad) {
        int g, n;
        float v = neg_inf();
        if (row_valid(a, lane, g, n)) {
            const uint64_t *src = a.lse + (size_t)(pc % kSlots) * a.rows_pad + lane;
            if ((uint32_t)(pend.lse_entry >> 32) != (uint32_t)(pc + 1) && *s_fail == 0) {
                unsigned spins = 0;
                do {
                    if (++spins > kSpinMax) { *s_fail = 1; break; }
                    pend.lse_entry = ld64(src);
                } while ((uint32_t)(pend.lse_entry >> 32) != (uint32_t)(pc + 1));
            }
            v = __uint_as_float((uint32_t)pend.lse_entry);
        }
        const int rho = lane & 31;
        cinit[(lane & ~31) + ((rho >> 2) & 1) * 16 + 4 * (rho >> 3) + (rho & 3)] = v;
    }
    lds_barrier();                                                            // B1

    // ---- S2: probability pass of phase pc ----
    if (pc >= 0 && pc < n_phases) {
        prob_pass<NB>(a, ring.kf[SLOT], q2, cinit, acc, hf, col);
        const PhaseId idc = phase_of(pc, a.n_kv_heads);
        if (idc.kv == a.n_kv_heads - 1 && (a.layer_agg == SP_LAYER_MEAN || idc.layer == a.n_layers - 1))
            close_layer<NB>(acc, a.c);
    }
    // ---- S3 + S4: lift K(it) into the ring slot just freed, statistics pass ----
    if (it < n_phases) {
#pragma unroll
        for (int s = 0; s < kNS; ++s) load_frag<kD>(kt, (wave * kNS + s) * 32 + col, hf, ring.kf[SLOT][s]);
        stats_pass(a, ring.kf[SLOT], q1, wstats[wave], n_valid, wave, hf, col);
    }
    lds_barrier();                                                            // B2

    // ---- S5: publish, then request what the next iteration needs ----
    if (it < n_phases && tid < a.rows_pad) {
        int g, n;
        if (row_valid(a, tid, g, n)) {
            float m = wstats[0][tid].x, l = wstats[0][tid].y;
#pragma unroll
            for (int ww = 1; ww < kFWaves; ++ww) lse_merge(m, l, wstats[ww][tid].x, wstats[ww][tid].y, a.c);
            const uint64_t bits = (uint64_t)__float_as_uint(m) | ((uint64_t)__float_as_uint(l) << 32) |
                                  ((uint64_t)((it / kSlots) & 1) << 63);
            st64(a.part + ((size_t)(it % kSlots) * a.rows_pad + tid) * a.n_wg + w, bits);
        }
    }
    if (wave == 1) {           // partials of the row this workgroup combines next iteration (phase it - 1)
        const int pn = clampi(it - 1, 0, n_phases - 1);
        const int r = min(duty_row_of(a, pn, w), a.rows_pad - 1);
        const uint64_t *src = a.part + ((size_t)(pn % kSlots) * a.rows_pad + r) * a.n_wg;
#pragma unroll
        for (int q = 0; q < 4; ++q) pend.duty[q] = ld64(src + min(lane + 64 * q, a.n_wg - 1));
    }
    if (wave == 0) {           // normalisers of the phase whose probability pass runs next iteration
        const int pn = clampi(pc + 1, 0, n_phases - 1);
        pend.lse_entry = ld64(a.lse + (size_t)(pn % kSlots) * a.rows_pad + min(lane, a.rows_pad - 1));
    }
    {
        const PhaseId id1 = phase_of(min(it + 1, n_phases - 1), a.n_kv_heads);
        issue_q_tile(q1, a, id1.layer, id1.kv, wave, lane);
        const PhaseId id2 = phase_of(clampi(pc + 1, 0, n_phases - 1), a.n_kv_heads);
        issue_q_tile(q2, a, id2.layer, id2.kv, wave, lane);
        // K two phases ahead; past the last phase a one-row dummy keeps the instruction count fixed
        const PhaseId id3 = phase_of(min(it + 2, n_phases - 1), a.n_kv_heads);
        issue_k_tile(kt, kp.p[id3.layer] + (int64_t)id3.kv * a.k_stride_head, a.k_stride_token,
                     (int64_t)w * kFTile, (it + 2 < n_phases) ? n_valid : 1, wave, lane);
    }
}

template <int NB>
__global__ __launch_bounds__(kFThreads, 2) void sp_fused_kernel(FusedArgs a, LayerPtrs kp)
{
    __shared__ u32x4 kt0[kFTile * kCH];
    __shared__ u32x4 kt1[kFTile * kCH];
    __shared__ u32x4 q1[kMaxRowsF * kCH];
    __shared__ u32x4 q2[kMaxRowsF * kCH];
    __shared__ float2 wstats[kFWaves][kMaxRowsF];
    __shared__ float cinit[kMaxRowsF];
    __shared__ int s_fail;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, hf = lane >> 5, col = lane & 31;
    const int w = blockIdx.x;
    const int n_phases = a.n_layers * a.n_kv_heads;
    const int64_t j0 = (int64_t)w * kFTile;
    const int n_valid = (int)((a.L - j0 < kFTile) ? a.L - j0 : kFTile);

    if (tid < kMaxRowsF) cinit[tid] = neg_inf();
    if (tid == 0) s_fail = 0;
    lds_barrier();

    Ring ring;
    Acc<NB> acc;
    Pending pend;
    pend.lse_entry = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) pend.duty[q] = 0;
#pragma unroll
    for (int s = 0; s < kNS; ++s) {
        acc.total[s] = 0.f;
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc.mx[s][b][e] = neg_inf();
    }

    // prologue: Q(0), K(0), K(1)
    issue_q_tile(q1, a, 0, 0, wave, lane);
    issue_k_tile(kt0, kp.p[0], a.k_stride_token, j0, n_valid, wave, lane);
    {
        const PhaseId id = phase_of(min(1, n_phases - 1), a.n_kv_heads);
        issue_k_tile(kt1, kp.p[id.layer] + (int64_t)id.kv * a.k_stride_head, a.k_stride_token, j0,
                     n_phases > 1 ? n_valid : 1, wave, lane);
    }

    // The body is unrolled six times so that the ring slot (it % 3) and the transit buffer (it % 2)
    // are compile-time; the trip count is rounded up, surplus iterations do no work but keep the
    // instruction stream uniform.
    const int n_iter = (n_phases + kLag + 5) / 6 * 6;
    for (int it0 = 0; it0 < n_iter; it0 += 6) {
#define SP_ITER(SLOT, BUF, OFF)                                                                           \
        iteration<NB, SLOT, BUF>(a, kp, it0 + OFF, n_phases, ring, acc, pend, kt0, kt1, q1, q2, wstats,   \
                                 cinit, &s_fail, n_valid);
        SP_ITER(0, 0, 0)
        SP_ITER(1, 1, 1)
        SP_ITER(2, 0, 2)
        SP_ITER(0, 1, 3)
        SP_ITER(1, 0, 4)
        SP_ITER(2, 1, 5)
#undef SP_ITER
    }
    vm_wait<0>();               // no direct-to-LDS load may outlive the workgroup
    lds_barrier();
    const bool failed = s_fail != 0;
    if (failed && tid == 0) __hip_atomic_store(a.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
    for (int s = 0; s < kNS; ++s) {
        const float both = acc.total[s] + __shfl_xor(acc.total[s], 32);
        const int key = (wave * kNS + s) * 32 + col;
        if (hf == 0 && key < n_valid) a.scores[j0 + key] = failed ? __builtin_nanf("") : both * a.out_scale;
    }
}

// Clears the exchange area: a zero sum marks a partial as not yet written and
// phase numbers start at 1, so zero normaliser entries are never taken as ready.
__global__ void sp_fused_clear_kernel(uint64_t *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0;
}

}  // namespace

namespace sp_fused {

size_t workspace_bytes(int rows_pad, int n_wg)
{
    return sp::align_up(sizeof(uint64_t) * ((size_t)kSlots * rows_pad * n_wg + (size_t)kSlots * rows_pad + 32), 256);
}

bool fits_one_per_cu()
{
    int n1 = 0, n2 = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n1, sp_fused_kernel<1>, kFThreads, 0) != hipSuccess) return false;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n2, sp_fused_kernel<2>, kFThreads, 0) != hipSuccess) return false;
    return n1 >= 1 && n2 >= 1;
}

sp_status launch(FusedArgs a, const LayerPtrs &kp, void *ws, hipStream_t st)
{
    uint64_t *base = static_cast<uint64_t *>(ws);
    const size_t n_part = (size_t)kSlots * a.rows_pad * a.n_wg, n_lse = (size_t)kSlots * a.rows_pad;
    a.part = base;
    a.lse = base + n_part;
    a.err = reinterpret_cast<uint32_t *>(base + n_part + n_lse);
    a.zeros = base + n_part + n_lse + 16;          // 128 bytes of zeros for padding query rows
    const size_t n_clear = n_part + n_lse + 32;
    hipLaunchKernelGGL(sp_fused_clear_kernel, dim3((unsigned)((n_clear + 255) / 256 > 1024 ? 1024 : (n_clear + 255) / 256)),
                       dim3(256), 0, st, base, n_clear);
    SP_HIP_CHECK(hipGetLastError());
    // Every workgroup must be resident for the exchange to make progress: one workgroup fits per
    // compute unit (LDS), so the grid may not exceed the number of compute units. All waits in the
    // kernel are bounded; should residency fail (the device shared with other work), the call ends
    // with NaN scores and the error word set instead of hanging.
    if (a.n_nblk == 1)
        hipLaunchKernelGGL(sp_fused_kernel<1>, dim3(a.n_wg), dim3(kFThreads), 0, st, a, kp);
    else
        hipLaunchKernelGGL(sp_fused_kernel<2>, dim3(a.n_wg), dim3(kFThreads), 0, st, a, kp);
    SP_HIP_CHECK(hipGetLastError());
    return SP_OK;
}

}  // namespace sp_fused

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
//    two transit buffers. K is wave-private: each wave loads, and later lifts
//    into MFMA fragments, its own 64 keys, so the K path needs no barrier. The
//    fragments of four phases live in registers (a ring of 4 x 32 VGPRs);
//  * a vector-memory instruction blocks its wave while the compute unit's memory
//    pipe is full, and the pipe drains at the unit's share of HBM bandwidth, so
//    the eight tile loads of an iteration are issued one by one between the
//    MFMA steps: while one wave waits for a slot the other waves compute;
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
constexpr int kTileInstr = kFTile / 64;   // tile-load instructions per wave per tile (8 rows each)
constexpr int kLag = 3;                   // phases between statistics and probability pass
constexpr int kRing = kLag + 1;           // fragment ring: phases it-3 .. it
constexpr int kSlots = sp_fused::kSlots;  // exchange ring depth
constexpr int kMaxRowsF = sp_fused::kMaxRows;   // 64 padded query rows per kv head
constexpr unsigned kSpinMax = 1u << 20;    // polls before a wait gives up (about a second)
constexpr int kDutyWave = 1;               // the wave that combines this workgroup's duty row
constexpr int kLseWave = 2;                // the wave that fetches the normalisers

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

// max(a, b, c); built without NaN honouring the compiler emits a single v_max3_f32 for it
__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

struct Ring {
    bf16x8 kf[kRing][kNS][kKS];           // K fragments of the phases in flight
};

// LDS reads of tiles filled by direct-to-LDS loads are written as asm blocks: the compiler cannot
// tell which in-flight load targets which buffer and would put a full vector-memory wait in front
// of every such read. The kernel waits (vm_wait + barrier) for exactly what it is about to read.
//
// Lifts this wave's 64 keys (two 32-key sub-tiles, four k-steps each) from a transit buffer.
__device__ __forceinline__ void lift_k_tile(const u32x4 *tile, int row0, int hf, bf16x8 (&f)[kNS][kKS])
{
    static_assert(kNS == 2 && kKS == 4, "layout of the asm block");
    const uint32_t base = (uint32_t)reinterpret_cast<uintptr_t>(SP_LPTR(tile));
    uint32_t ad[kKS];
#pragma unroll
    for (int t = 0; t < kKS; ++t) ad[t] = base + 16u * (uint32_t)lds_slot<kD>(row0, 2 * t + hf);
    u32x4 r[kNS][kKS];
    // sub-tile 1 starts 32 rows = 4096 bytes later; (row >> 1) & 7 and hence the swizzle are the same
    __asm__ volatile(
        "ds_read_b128 %0, %8\n\t"
        "ds_read_b128 %1, %9\n\t"
        "ds_read_b128 %2, %10\n\t"
        "ds_read_b128 %3, %11\n\t"
        "ds_read_b128 %4, %8 offset:4096\n\t"
        "ds_read_b128 %5, %9 offset:4096\n\t"
        "ds_read_b128 %6, %10 offset:4096\n\t"
        "ds_read_b128 %7, %11 offset:4096\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(r[0][0]), "=&v"(r[0][1]), "=&v"(r[0][2]), "=&v"(r[0][3]),
          "=&v"(r[1][0]), "=&v"(r[1][1]), "=&v"(r[1][2]), "=&v"(r[1][3])
        : "v"(ad[0]), "v"(ad[1]), "v"(ad[2]), "v"(ad[3])
        : "memory");
#pragma unroll
    for (int s = 0; s < kNS; ++s)
#pragma unroll
        for (int t = 0; t < kKS; ++t) f[s][t] = __builtin_bit_cast(bf16x8, r[s][t]);
}

// Fragments of one 32-row block of a Q tile.
__device__ __forceinline__ void lift_q_block(const u32x4 *tile, int row, int hf, bf16x8 (&f)[kKS])
{
    static_assert(kKS == 4, "layout of the asm block");
    const uint32_t base = (uint32_t)reinterpret_cast<uintptr_t>(SP_LPTR(tile));
    uint32_t ad[kKS];
#pragma unroll
    for (int t = 0; t < kKS; ++t) ad[t] = base + 16u * (uint32_t)lds_slot<kD>(row, 2 * t + hf);
    u32x4 r[kKS];
    __asm__ volatile(
        "ds_read_b128 %0, %4\n\t"
        "ds_read_b128 %1, %5\n\t"
        "ds_read_b128 %2, %6\n\t"
        "ds_read_b128 %3, %7\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3])
        : "v"(ad[0]), "v"(ad[1]), "v"(ad[2]), "v"(ad[3])
        : "memory");
#pragma unroll
    for (int t = 0; t < kKS; ++t) f[t] = __builtin_bit_cast(bf16x8, r[t]);
}

// A plain LDS store, opaque to the compiler for the same reason (ordered by the next barrier).
__device__ __forceinline__ void lds_store_f32(float *p, float v)
{
    const uint32_t ad = (uint32_t)reinterpret_cast<uintptr_t>(SP_LPTR(p));
    __asm__ volatile("ds_write_b32 %0, %1" : : "v"(ad), "v"(v) : "memory");
}

__device__ __forceinline__ float2 lds_load_f2(const float2 *p)
{
    const uint32_t ad = (uint32_t)reinterpret_cast<uintptr_t>(SP_LPTR(p));
    float2 v;
    __asm__ volatile("ds_read_b64 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(v) : "v"(ad) : "memory");
    return v;
}

// Butterfly reductions with data-parallel-primitive moves: after the three steps every lane of an
// aligned group of 8 holds the group's result; one more step extends it to the row of 16. Every
// lane adds the same two operands in either order, so the results are identical across lanes.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
constexpr int kDppXor1 = 0xB1;          // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;          // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;   // lane i <- lane 7 - i within groups of 8
constexpr int kDppMirror = 0x140;       // lane i <- lane 15 - i within rows of 16

__device__ __forceinline__ float group8_max(float v)
{
    v = fmaxf(v, dpp_move<kDppXor1>(v));
    v = fmaxf(v, dpp_move<kDppXor2>(v));
    return fmaxf(v, dpp_move<kDppHalfMirror>(v));
}
__device__ __forceinline__ float group8_sum(float v)
{
    v += dpp_move<kDppXor1>(v);
    v += dpp_move<kDppXor2>(v);
    return v + dpp_move<kDppHalfMirror>(v);
}
__device__ __forceinline__ float lane_value(float v, int lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}
__device__ __forceinline__ float wave_max(float v)
{
    v = group8_max(v);
    v = fmaxf(v, dpp_move<kDppMirror>(v));
    return fmaxf(fmaxf(lane_value(v, 0), lane_value(v, 16)), fmaxf(lane_value(v, 32), lane_value(v, 48)));
}
__device__ __forceinline__ float wave_sum(float v)
{
    v = group8_sum(v);
    v += dpp_move<kDppMirror>(v);
    return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}

struct PhaseId { int layer, kv; };
__device__ __forceinline__ PhaseId phase_of(int p, int n_kv) { PhaseId r; r.layer = p / n_kv; r.kv = p - r.layer * n_kv; return r; }

// padded query row -> (group head, lookahead row); see the row order in sp_score.hip
template <int NB>
__device__ __forceinline__ bool row_valid(const FusedArgs &a, int row, int &g, int &n)
{
    const int blk = row >> 5, rho = row & 31;
    const int gblk = blk / NB, nblk = blk - gblk * NB;
    g = 4 * gblk + (rho >> 3);
    n = 8 * nblk + (rho & 7);
    return g < a.group && n < a.n_q;
}

// One wave instruction moves 64 chunks = 8 key rows (1 KB, contiguous in HBM when keys are
// contiguous); a wave's 64 rows take eight of them. The address is a uniform base plus a 32-bit
// per-lane byte offset, so no address registers stay live between instructions.
struct KIssue {
    u32x4 *tile;              // transit buffer being refilled
    const uint16_t *base;     // first key of this workgroup in the (layer, kv head) being fetched (uniform)
    uint32_t stride_bytes;    // bytes between consecutive keys
    int n_valid, wave, lane;
};

// Issues instructions first .. first+COUNT-1 of the tile (first and COUNT compile-time at call sites).
template <int COUNT>
__device__ __forceinline__ void k_issue(const KIssue &ki, int first)
{
#pragma unroll
    for (int i = 0; i < COUNT; ++i) {
        const int idx = first + i;
        int row = ki.wave * 64 + 8 * idx + (ki.lane >> 3);
        const uint32_t chunk = (uint32_t)((ki.lane & 7) ^ ((row >> 1) & 7));
        row = row < ki.n_valid ? row : ki.n_valid - 1;        // tail rows repeat the last valid key
        const uint32_t off = (uint32_t)row * ki.stride_bytes + chunk * 16u;
        const char *src = reinterpret_cast<const char *>(ki.base) + off;
        __builtin_amdgcn_global_load_lds(SP_GPTR(src), SP_LPTR(ki.tile + (ki.wave * 64 + 8 * idx) * kCH), 16, 0, 0);
    }
}

// Each wave loads eight rows (one instruction) of a Q tile of one (layer, kv head), in the padded
// row order; padding rows read a zero line kept in the workspace.
template <int NB>
__device__ __forceinline__ void issue_q_slice(u32x4 *qt, const FusedArgs &a, int layer, int kv, int wave, int lane)
{
    const int row = wave * 8 + (lane >> 3);
    int g, n;
    const uint16_t *src = reinterpret_cast<const uint16_t *>(a.zeros) + (lane & 7) * 8;
    if (row < a.rows_pad && row_valid<NB>(a, row, g, n)) {
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

// ---- probability pass of one phase from the fragment ring; tile loads are issued between the MFMA steps ----
template <int NB, int GB>
__device__ __forceinline__ void prob_pass(const bf16x8 (&kf)[kNS][kKS], const u32x4 *q2, const float *cinit,
                                          Acc<NB> &acc, int hf, int col, const KIssue &ki, int first)
{
    constexpr int kPerStep = (kTileInstr / 2) / (NB * GB * kNS);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
        for (int gb = 0; gb < GB; ++gb) {
            const int blk = gb * NB + nb;
            bf16x8 qf[kKS];
            lift_q_block(q2, blk * 32 + col, hf, qf);
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
                // d[r]: group head r/4, lookahead row 8*nb + 4*hf + r%4, key (wave*2+s)*32 + col
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    acc.mx[s][nb][e] = max3(max3(d[e], d[4 + e], d[8 + e]), d[12 + e], acc.mx[s][nb][e]);
                k_issue<kPerStep>(ki, first + ((nb * GB + gb) * kNS + s) * kPerStep);
                __builtin_amdgcn_sched_barrier(0);
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
template <int NBLK>
__device__ __forceinline__ void stats_pass(float c, const bf16x8 (&kf)[kNS][kKS], const u32x4 *q1,
                                           float2 *wstats_wave, int n_valid, int wave, int hf, int col,
                                           const KIssue &ki)
{
    constexpr int kPerStep = (kTileInstr / 2) / (NBLK * kNS);   // tile-load instructions issued after each MFMA step
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) {
        bf16x8 qf[kKS];
        lift_q_block(q1, blk * 32 + col, hf, qf);
        float m = neg_inf(), l = 0.f;
#pragma unroll
        for (int s = 0; s < kNS; ++s) {
            f32x16 d = {0.f};
#pragma unroll
            for (int t = 0; t < kKS; ++t) d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s][t], qf[t], d, 0, 0, 0);
            // d[r]: key (wave*2+s)*32 + 8*(r/4) + 4*hf + r%4 of the tile, query row blk*32 + col
            const int left = n_valid - (wave * kNS + s) * 32;
            if (left >= 32) {
                float mn = max3(m, d[0], d[1]);      // running maximum including these 16 logits
#pragma unroll
                for (int r = 2; r < 16; r += 2) mn = max3(mn, d[r], d[r + 1]);
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
            k_issue<kPerStep>(ki, (blk * kNS + s) * kPerStep);
            __builtin_amdgcn_sched_barrier(0);
        }
        const float m2 = __shfl_xor(m, 32), l2 = __shfl_xor(l, 32);
        lse_merge(m, l, m2, l2, c);
        if (hf == 0) wstats_wave[blk * 32 + col] = make_float2(m, l);
    }
}

// Exchange data requested with direct-to-LDS loads lands in two small staging areas private to
// the exchange wave: xduty holds the n_wg partials of the duty row (entry e at byte 8e), xlse the
// normaliser entries of one phase. Reading them back in asm keeps the compiler from waiting for
// every vector-memory operation in flight.
struct DutyEntries { uint64_t e[4]; };     // entries lane, lane + 64, lane + 128, lane + 192

__device__ __forceinline__ DutyEntries read_duty_staging(const u32x4 *xduty, int lane)
{
    const uint32_t ad = (uint32_t)reinterpret_cast<uintptr_t>(SP_LPTR(xduty)) + 8u * (uint32_t)lane;
    DutyEntries d;
    __asm__ volatile(
        "ds_read_b64 %0, %4\n\t"
        "ds_read_b64 %1, %4 offset:512\n\t"
        "ds_read_b64 %2, %4 offset:1024\n\t"
        "ds_read_b64 %3, %4 offset:1536\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(d.e[0]), "=&v"(d.e[1]), "=&v"(d.e[2]), "=&v"(d.e[3])
        : "v"(ad)
        : "memory");
    return d;
}

__device__ __forceinline__ uint64_t read_lse_staging(const u32x4 *xlse, int lane)
{
    const uint32_t ad = (uint32_t)reinterpret_cast<uintptr_t>(SP_LPTR(xlse)) + 8u * (uint32_t)lane;
    uint64_t v;
    __asm__ volatile("ds_read_b64 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(v) : "v"(ad) : "memory");
    return v;
}

// Direct-to-LDS load of 64 x 16 bytes: the 16-byte pairs first .. first+63 of a row of 8-byte
// entries (row 16-byte aligned) that holds `pairs` pairs; lanes beyond the row repeat its last pair.
// The load bypasses the non-coherent cache levels like the atomic loads of the retry paths do.
__device__ __forceinline__ void stage_entries(u32x4 *dst, const uint64_t *row, int first, int pairs, int lane)
{
    constexpr int kDeviceScope = 16;      // the sc1 bit of the cache-policy operand
    const uint64_t *p = row + 2 * min(first + lane, pairs - 1);
    __builtin_amdgcn_global_load_lds(SP_GPTR(p), SP_LPTR(dst), 16, 0, kDeviceScope);
}

// A partial is ready when it carries the parity of this use of its slot and a non-zero sum.
// Entries beyond the last workgroup do not exist and count as ready.
__device__ __forceinline__ bool duty_ready(const DutyEntries &d, uint32_t par, int lane, int n_wg)
{
    uint32_t ok = 1u;           // branch-free: one straight-line test of the four entries
#pragma unroll
    for (int q = 0; q < 4; ++q)
        ok &= (uint32_t)(lane + 64 * q >= n_wg) |
              ((uint32_t)((uint32_t)(d.e[q] >> 63) == par) & (uint32_t)(((d.e[q] >> 32) & 0x7fffffffu) != 0));
    return ok != 0;
}

// Row of phase p that workgroup w combines (>= rows_pad: none). Rows rotate over the workgroups.
__device__ __forceinline__ int duty_row_of(const FusedArgs &a, int p, int w)
{
    const int first = (int)(((uint32_t)p * (uint32_t)a.rows_pad) % (uint32_t)a.n_wg);
    const int r = w - first;
    return r < 0 ? r + a.n_wg : r;
}

// One iteration `it` of the software pipeline. Per wave, in program order:
//   top     wait for everything but the four newest loads; one wave combines the duty row of phase
//           it-2 and publishes its normaliser, another puts the normalisers of phase it-3 into LDS
//   B1
//   lift    this wave's slice of Q(it-2) for the next iteration's probability pass; this wave's keys
//           of K(it) from transit buffer it%2 into ring slot it%4
//   stats   statistics pass of phase it; first four loads of K(it+2) into the buffer just emptied
//   B2
//   mid     every wave: publish this workgroup's partials of eight rows of phase it, its slice of
//           Q(it+1); the two exchange waves request the partials of phase it-1 (duty row) and the
//           normalisers of phase it-2
//   prob    probability pass of phase it-3; last four loads of K(it+2)
// The four newest vector-memory operations of a wave are therefore always K-tile loads whose data
// is not needed before the iteration after next; everything older has landed after vm_wait<4>.
template <int NB, int GB, int SLOT, int BUF>
__device__ __forceinline__ void iteration(const FusedArgs &a, const LayerPtrs &kp, int it, int n_phases, Ring &ring,
                                          Acc<NB> &acc, u32x4 *xduty, u32x4 *xlse, u32x4 *kt0, u32x4 *kt1, u32x4 *q1, u32x4 *q2a,
                                          u32x4 *q2b, float2 (*wstats)[kMaxRowsF], float (*cinit2)[kMaxRowsF],
                                          int *s_fail, int n_valid)
{
    // Lane-derived LDS and global offsets are recomputed every iteration instead of being kept in
    // registers across the whole loop (the opaque copy stops the compiler from hoisting them).
    int tid = threadIdx.x;
    __asm__ volatile("" : "+v"(tid));
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, hf = lane >> 5, col = lane & 31;
    const int w = blockIdx.x;
    u32x4 *kt = BUF ? kt1 : kt0;
    u32x4 *q2 = BUF ? q2b : q2a;          // Q of phase it-3; the other buffer receives Q of phase it-2
    u32x4 *q2_next = BUF ? q2a : q2b;
    float *cinit = cinit2[BUF];           // double-buffered: waves may still read the other one
    const int pc = it - kLag;             // phase whose probability pass runs in this iteration
    const int pd = it - 2;                // phase whose duty loads were issued last iteration
    const bool do_prob = pc >= 0 && pc < n_phases, do_stats = it < n_phases;

    // ---- top ----
    vm_wait<kTileInstr / 2>();
    if (wave == kDutyWave) {
        if (pd >= 0 && pd < n_phases) {
            const int duty_row = duty_row_of(a, pd, w);
            int g, n;
            if (duty_row < a.rows_pad && row_valid<NB>(a, duty_row, g, n)) {
                const uint32_t par = (uint32_t)(pd / kSlots) & 1u;
                const uint64_t *src = a.part + ((size_t)(pd % kSlots) * a.rows_pad + duty_row) * a.part_stride;
                // fast path: the partials requested last iteration are all there; otherwise poll (bounded)
                DutyEntries de = read_duty_staging(xduty, lane);
                if (__any(!duty_ready(de, par, lane, a.n_wg)) && *s_fail == 0) {
                    unsigned spins = 0;
                    do {
                        if (++spins > kSpinMax) { *s_fail = 1; break; }
#pragma unroll
                        for (int q = 0; q < 4; ++q) de.e[q] = ld64(src + min(lane + 64 * q, a.n_wg - 1));
                    } while (__any(!duty_ready(de, par, lane, a.n_wg)));
                }
                // maximum first, then one exponential per partial: short dependency chains, fixed order
                float pm[4], pl[4], m = neg_inf();
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const bool valid = lane + 64 * q < a.n_wg;
                    pm[q] = valid ? __uint_as_float((uint32_t)de.e[q]) : neg_inf();
                    pl[q] = valid ? __uint_as_float((uint32_t)(de.e[q] >> 32) & 0x7fffffffu) : 0.f;
                    m = fmaxf(m, pm[q]);
                }
                m = wave_max(m);
                float l = 0.f;
#pragma unroll
                for (int q = 0; q < 4; ++q) l += pl[q] * fast_exp2((pm[q] - m) * a.c);
                l = wave_sum(l);
                if (lane == 0) {
                    const float v = -(m + fast_log2(l) * a.inv_c);
                    st64(a.lse + (size_t)(pd % kSlots) * a.rows_pad + duty_row,
                         (uint64_t)__float_as_uint(v) | ((uint64_t)(uint32_t)(pd + 1) << 32));
                }
            }
        }
    } else if (wave == kLseWave) {
        if (do_prob && lane < a.rows_pad) {
            int g, n;
            float v = neg_inf();
            if (row_valid<NB>(a, lane, g, n)) {
                const uint64_t *src = a.lse + (size_t)(pc % kSlots) * a.rows_pad + lane;
                uint64_t entry = read_lse_staging(xlse, lane);
                if ((uint32_t)(entry >> 32) != (uint32_t)(pc + 1) && *s_fail == 0) {
                    unsigned spins = 0;
                    do {
                        if (++spins > kSpinMax) { *s_fail = 1; break; }
                        entry = ld64(src);
                    } while ((uint32_t)(entry >> 32) != (uint32_t)(pc + 1));
                }
                v = __uint_as_float((uint32_t)entry);
            }
            const int rho = lane & 31;
            lds_store_f32(cinit + (lane & ~31) + ((rho >> 2) & 1) * 16 + 4 * (rho >> 3) + (rho & 3), v);
        }
    }
    lds_barrier();                                                            // B1: K(it), Q tiles, cinit ready

    // ---- Q of the next probability pass, lift, statistics pass; first half of the loads of K(it+2) ----
    {
        const PhaseId id2 = phase_of(clampi(pc + 1, 0, n_phases - 1), a.n_kv_heads);
        issue_q_slice<NB>(q2_next, a, id2.layer, id2.kv, wave, lane);
    }
    KIssue ki;
    {
        const PhaseId id3 = phase_of(min(it + 2, n_phases - 1), a.n_kv_heads);
        ki.tile = kt;
        ki.base = kp.p[id3.layer] + (int64_t)id3.kv * a.k_stride_head + (int64_t)w * kFTile * a.k_stride_token;
        ki.stride_bytes = (uint32_t)a.k_stride_token * 2u;
        ki.n_valid = (it + 2 < n_phases) ? n_valid : 1;     // past the last phase: a one-row dummy keeps the count fixed
        ki.wave = wave; ki.lane = lane;
    }
    if (do_stats) {
        lift_k_tile(kt, wave * kNS * 32 + col, hf, ring.kf[SLOT]);
        stats_pass<NB * GB>(a.c, ring.kf[SLOT], q1, wstats[wave], n_valid, wave, hf, col, ki);
    } else {
        k_issue<kTileInstr / 2>(ki, 0);
    }
    lds_barrier();                                                            // B2: wstats complete, q1 free

    // ---- mid: exchange traffic and Q of the next statistics pass, ahead of the remaining K loads ----
    if (do_stats) {
        // every wave combines the eight per-wave statistics of eight rows (lane = row x source wave)
        // and publishes them: maximum first, then one exponential per source
        const int row = wave * 8 + (lane >> 3);
        const float2 st = lds_load_f2(&wstats[lane & 7][row]);
        const float m = group8_max(st.x);
        const float l = group8_sum(st.y * fast_exp2((st.x - m) * a.c));
        int g, n;
        if ((lane & 7) == 0 && row < a.rows_pad && row_valid<NB>(a, row, g, n)) {
            const uint64_t bits = (uint64_t)__float_as_uint(m) | ((uint64_t)__float_as_uint(l) << 32) |
                                  ((uint64_t)((it / kSlots) & 1) << 63);
            st64(a.part + ((size_t)(it % kSlots) * a.rows_pad + row) * a.part_stride + w, bits);
        }
    }
    if (wave == kDutyWave) {        // partials of the row this workgroup combines at the next top (phase it - 1)
        const int pn = clampi(it - 1, 0, n_phases - 1);
        const int r = min(duty_row_of(a, pn, w), a.rows_pad - 1);
        const uint64_t *src = a.part + ((size_t)(pn % kSlots) * a.rows_pad + r) * a.part_stride;
        stage_entries(xduty, src, 0, a.part_stride / 2, lane);
        stage_entries(xduty + 64, src, 64, a.part_stride / 2, lane);
    } else if (wave == kLseWave) {  // normalisers of the phase whose probability pass runs next iteration
        const int pn = clampi(pc + 1, 0, n_phases - 1);
        stage_entries(xlse, a.lse + (size_t)(pn % kSlots) * a.rows_pad, 0, a.rows_pad / 2, lane);
    }
    {
        const PhaseId id1 = phase_of(min(it + 1, n_phases - 1), a.n_kv_heads);
        issue_q_slice<NB>(q1, a, id1.layer, id1.kv, wave, lane);
    }

    // ---- probability pass of phase pc; second half of the loads of K(it+2) ----
    if (do_prob) {
        prob_pass<NB, GB>(ring.kf[(SLOT + 1) % kRing], q2, cinit, acc, hf, col, ki, kTileInstr / 2);
        const PhaseId idc = phase_of(pc, a.n_kv_heads);
        if (idc.kv == a.n_kv_heads - 1 && (a.layer_agg == SP_LAYER_MEAN || idc.layer == a.n_layers - 1))
            close_layer<NB>(acc, a.c);
    } else {
        k_issue<kTileInstr / 2>(ki, kTileInstr / 2);
    }
}

template <int NB, int GB>
__global__ __launch_bounds__(kFThreads, 2) void sp_fused_kernel(FusedArgs a, LayerPtrs kp)
{
    __shared__ u32x4 kt0[kFTile * kCH];
    __shared__ u32x4 kt1[kFTile * kCH];
    __shared__ u32x4 q1[kMaxRowsF * kCH];
    __shared__ u32x4 q2a[kMaxRowsF * kCH];
    __shared__ u32x4 q2b[kMaxRowsF * kCH];
    __shared__ float2 wstats[kFWaves][kMaxRowsF];
    __shared__ float cinit2[2][kMaxRowsF];
    __shared__ u32x4 xduty[128];             // partials of the duty row, 256 entries
    __shared__ u32x4 xlse[64];               // normaliser entries of one phase (64 used, the load moves 128)
    __shared__ int s_fail;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, hf = lane >> 5, col = lane & 31;
    const int w = blockIdx.x;
    const int n_phases = a.n_layers * a.n_kv_heads;
    const int64_t j0 = (int64_t)w * kFTile;
    const int n_valid = (int)((a.L - j0 < kFTile) ? a.L - j0 : kFTile);

    if (tid < 2 * kMaxRowsF) cinit2[tid / kMaxRowsF][tid % kMaxRowsF] = neg_inf();
    if (tid == 0) s_fail = 0;
    lds_barrier();

    Ring ring;
    Acc<NB> acc;
#pragma unroll
    for (int s = 0; s < kNS; ++s) {
        acc.total[s] = 0.f;
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc.mx[s][b][e] = neg_inf();
    }

    // prologue: this wave's slice of Q(0), then its rows of K(0) and K(1)
    issue_q_slice<NB>(q1, a, 0, 0, wave, lane);
    {
        KIssue ki;
        ki.stride_bytes = (uint32_t)a.k_stride_token * 2u; ki.wave = wave; ki.lane = lane;
        ki.tile = kt0; ki.base = kp.p[0] + j0 * a.k_stride_token; ki.n_valid = n_valid;
        k_issue<kTileInstr>(ki, 0);
        const PhaseId id = phase_of(min(1, n_phases - 1), a.n_kv_heads);
        ki.tile = kt1; ki.base = kp.p[id.layer] + (int64_t)id.kv * a.k_stride_head + j0 * a.k_stride_token;
        ki.n_valid = n_phases > 1 ? n_valid : 1;
        k_issue<kTileInstr>(ki, 0);
    }

    // The body is unrolled four times so that the ring slot (it % 4) and the transit buffer (it % 2)
    // are compile-time; the trip count is rounded up, surplus iterations do no work but keep the
    // instruction stream uniform.
    const int n_iter = (n_phases + kLag + 3) / 4 * 4;
    for (int it0 = 0; it0 < n_iter; it0 += 4) {
#define SP_ITER(SLOT, BUF, OFF)                                                                               \
        iteration<NB, GB, SLOT, BUF>(a, kp, it0 + OFF, n_phases, ring, acc, xduty, xlse, kt0, kt1, q1, q2a, q2b,     \
                                     wstats, cinit2, &s_fail, n_valid);
        SP_ITER(0, 0, 0)
        SP_ITER(1, 1, 1)
        SP_ITER(2, 0, 2)
        SP_ITER(3, 1, 3)
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
        if (hf == 0 && key < n_valid) a.scores[j0 + key] = failed ? __uint_as_float(0x7fc00000u) : both * a.out_scale;   // quiet NaN marks a failed call
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

// Rows of partials start on 16-byte boundaries.
static int part_stride(int n_wg) { return (n_wg + 1) & ~1; }

size_t workspace_bytes(int rows_pad, int n_wg)
{
    return sp::align_up(sizeof(uint64_t) * ((size_t)kSlots * rows_pad * part_stride(n_wg) + (size_t)kSlots * rows_pad + 32), 256);
}

bool fits_one_per_cu()
{
    int n1 = 0, n2 = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n1, sp_fused_kernel<1, 1>, kFThreads, 0) != hipSuccess) return false;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n2, sp_fused_kernel<2, 1>, kFThreads, 0) != hipSuccess) return false;
    return n1 >= 1 && n2 >= 1;
}

sp_status launch(FusedArgs a, const LayerPtrs &kp, void *ws, hipStream_t st)
{
    uint64_t *base = static_cast<uint64_t *>(ws);
    a.part_stride = part_stride(a.n_wg);
    const size_t n_part = (size_t)kSlots * a.rows_pad * a.part_stride, n_lse = (size_t)kSlots * a.rows_pad;
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
    if (a.n_nblk == 2 && a.n_gblk == 1)
        hipLaunchKernelGGL((sp_fused_kernel<2, 1>), dim3(a.n_wg), dim3(kFThreads), 0, st, a, kp);
    else if (a.n_nblk == 1 && a.n_gblk == 2)
        hipLaunchKernelGGL((sp_fused_kernel<1, 2>), dim3(a.n_wg), dim3(kFThreads), 0, st, a, kp);
    else if (a.n_nblk == 1 && a.n_gblk == 1)
        hipLaunchKernelGGL((sp_fused_kernel<1, 1>), dim3(a.n_wg), dim3(kFThreads), 0, st, a, kp);
    else
        return sp::fail(SP_ERR_UNSUPPORTED, "fused score kernel: %d x %d row blocks", a.n_nblk, a.n_gblk);
    SP_HIP_CHECK(hipGetLastError());
    return SP_OK;
}

}  // namespace sp_fused

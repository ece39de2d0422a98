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
//  * tiles stream HBM -> LDS with direct-to-LDS loads about one and a half
//    phases ahead. K is wave-private: each wave loads its own 64 keys, in two
//    32-key sub-tiles, into a ring of three sub-tile slots, and later lifts them
//    into MFMA fragments, so the K path needs no barrier. The fragments of four
//    phases live in registers (a ring of 4 x 32 VGPRs);
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
//    lookahead rows and layers in registers. Scores are stored once at the end;
//  * Q tiles, per-wave statistics and accumulator seeds are double-buffered in
//    LDS so that one workgroup barrier per phase orders everything shared.
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
constexpr int kSubInstr = 4;              // tile-load instructions per sub-tile (8 rows, 1 KB each)
constexpr int kSubSlots = 3;              // sub-tile slots in a wave's transit ring
constexpr int kSubChunks = 32 * kCH;      // 16-byte chunks per sub-tile slot
constexpr int kLag = 3;                   // phases between statistics and probability pass
constexpr int kRing = kLag + 1;           // fragment ring: four phases
constexpr int kSlots = sp_fused::kSlots;  // exchange ring depth
constexpr int kMaxRowsF = sp_fused::kMaxRows;   // 64 padded query rows per kv head
constexpr unsigned kSpinMax = 1u << 20;    // polls before a wait gives up (about a second)
constexpr int kPubWave = 0;                // the wave that publishes this workgroup's partials
constexpr int kDutyWave = 1;               // the wave that combines this workgroup's duty rows
constexpr int kDutyRows = 4;               // consecutive query rows one duty covers (32 bytes per source workgroup)
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

// All LDS traffic of the main loop is written as asm: the compiler cannot tell which in-flight
// direct-to-LDS load targets which buffer and would put a full vector-memory wait in front of
// LDS accesses it can see. The kernel waits (vm_wait, barrier) for exactly what it is about to read.
__device__ __forceinline__ uint32_t lds_addr(const void *p) { return (uint32_t)reinterpret_cast<uintptr_t>(SP_LPTR(p)); }

// MFMA fragments of 32 rows of a swizzled 64-wide bf16 tile: lane (col, hf) takes row `row`,
// 16-byte chunks 2t + hf.
__device__ __forceinline__ void lift_block(const u32x4 *tile, int row, int hf, bf16x8 (&f)[kKS])
{
    static_assert(kKS == 4, "layout of the asm block");
    const uint32_t base = lds_addr(tile);
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

__device__ __forceinline__ void lds_store_f32(float *p, float v)
{
    __asm__ volatile("ds_write_b32 %0, %1" : : "v"(lds_addr(p)), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_store_f2(float2 *p, float2 v)
{
    __asm__ volatile("ds_write_b64 %0, %1" : : "v"(lds_addr(p)), "v"(v) : "memory");
}
__device__ __forceinline__ float2 lds_load_f2(const float2 *p)
{
    float2 v;
    __asm__ volatile("ds_read_b64 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(v) : "v"(lds_addr(p)) : "memory");
    return v;
}
// Sixteen consecutive floats (64-byte aligned).
__device__ __forceinline__ f32x16 lds_load_f16(const float *p)
{
    typedef __attribute__((ext_vector_type(4))) float f32x4;
    const uint32_t ad = lds_addr(p);
    f32x4 r[4];
    __asm__ volatile(
        "ds_read_b128 %0, %4\n\t"
        "ds_read_b128 %1, %4 offset:16\n\t"
        "ds_read_b128 %2, %4 offset:32\n\t"
        "ds_read_b128 %3, %4 offset:48\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3])
        : "v"(ad)
        : "memory");
    f32x16 o;
#pragma unroll
    for (int v = 0; v < 4; ++v) { o[4 * v] = r[v].x; o[4 * v + 1] = r[v].y; o[4 * v + 2] = r[v].z; o[4 * v + 3] = r[v].w; }
    return o;
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
// contiguous); a 32-key sub-tile takes four of them. The address is a uniform base plus a 32-bit
// per-lane byte offset, so no address registers stay live between instructions.
struct KIssue {
    u32x4 *slot;              // sub-tile slot being refilled (this wave's)
    const uint16_t *base;     // first key of this workgroup in the (layer, kv head) being fetched (uniform)
    uint32_t stride_bytes;    // bytes between consecutive keys
    int row0;                 // first key of the sub-tile within the workgroup's tile
    int n_valid, lane;
};

// Issues instructions first .. first+COUNT-1 of the sub-tile (first and COUNT compile-time at call sites).
template <int COUNT>
__device__ __forceinline__ void k_issue(const KIssue &ki, int first)
{
#pragma unroll
    for (int i = 0; i < COUNT; ++i) {
        const int idx = first + i;
        const int r = 8 * idx + (ki.lane >> 3);               // row within the sub-tile
        const uint32_t chunk = (uint32_t)((ki.lane & 7) ^ ((r >> 1) & 7));
        int row = ki.row0 + r;
        row = row < ki.n_valid ? row : ki.n_valid - 1;        // tail rows repeat the last valid key
        const uint32_t off = (uint32_t)row * ki.stride_bytes + chunk * 16u;
        const char *src = reinterpret_cast<const char *>(ki.base) + off;
        __builtin_amdgcn_global_load_lds(SP_GPTR(src), SP_LPTR(ki.slot + 8 * idx * kCH), 16, 0, 0);
    }
}

// Sub-tile s2 of phase p lives in slot (2p + s2) mod 3 of its wave's transit ring.
__device__ __forceinline__ u32x4 *sub_slot(u32x4 *kring, int wave, int p, int s2)
{
    return kring + (wave * kSubSlots + (2 * p + s2) % kSubSlots) * kSubChunks;
}

__device__ __forceinline__ KIssue k_issue_setup(const FusedArgs &a, const LayerPtrs &kp, u32x4 *kring, int p, int s2,
                                                int n_phases, int n_valid, int wave, int lane)
{
    const PhaseId id = phase_of(min(p, n_phases - 1), a.n_kv_heads);
    KIssue ki;
    ki.slot = sub_slot(kring, wave, p, s2);
    ki.base = kp.p[id.layer] + (int64_t)id.kv * a.k_stride_head + (int64_t)blockIdx.x * kFTile * a.k_stride_token;
    ki.stride_bytes = (uint32_t)a.k_stride_token * 2u;
    ki.row0 = wave * 64 + s2 * 32;
    ki.n_valid = p < n_phases ? n_valid : 1;      // past the last phase: a one-row dummy keeps the count fixed
    ki.lane = lane;
    return ki;
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
                                          Acc<NB> &acc, int hf, int col, const KIssue &ki)
{
    constexpr int kPerStep = kSubInstr / (NB * GB * kNS);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
        for (int gb = 0; gb < GB; ++gb) {
            const int blk = gb * NB + nb;
            bf16x8 qf[kKS];
            lift_block(q2, blk * 32 + col, hf, qf);
            const f32x16 ci = lds_load_f16(cinit + blk * 32 + hf * 16);
#pragma unroll
            for (int s = 0; s < kNS; ++s) {
                f32x16 d = ci;
#pragma unroll
                for (int t = 0; t < kKS; ++t) d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[t], kf[s][t], d, 0, 0, 0);
                // d[r]: group head r/4, lookahead row 8*nb + 4*hf + r%4, key (wave*2+s)*32 + col
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    acc.mx[s][nb][e] = max3(max3(d[e], d[4 + e], d[8 + e]), d[12 + e], acc.mx[s][nb][e]);
                k_issue<kPerStep>(ki, ((nb * GB + gb) * kNS + s) * kPerStep);
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
    constexpr int kPerStep = kSubInstr / (NBLK * kNS);   // tile-load instructions issued after each MFMA step
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) {
        bf16x8 qf[kKS];
        lift_block(q1, blk * 32 + col, hf, qf);
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
        if (hf == 0) lds_store_f2(wstats_wave + blk * 32 + col, make_float2(m, l));
    }
}

// Exchange data requested with direct-to-LDS loads lands in two small staging areas, each private
// to one wave. Partials are stored workgroup-major, part[slot][workgroup][row], so that a workgroup
// publishes all its rows with one contiguous store; a duty covers kDutyRows consecutive rows, i.e.
// one 32-byte piece of every workgroup's line. xduty receives them as 16-byte pairs of rows:
// chunk (2q + h) * 64 + lane holds rows 2h and 2h+1 of the block from workgroup lane + 64q.
struct DutyBlock { uint64_t e[kDutyRows][4]; };     // [row of the block][workgroup lane + 64q]

__device__ __forceinline__ DutyBlock read_duty_staging(const u32x4 *xduty, int lane)
{
    static_assert(kDutyRows == 4, "layout of the asm block");
    typedef __attribute__((ext_vector_type(2))) uint64_t u64x2;
    const uint32_t ad = lds_addr(xduty) + 16u * (uint32_t)lane;
    u64x2 r[8];
    __asm__ volatile(
        "ds_read_b128 %0, %8\n\t"
        "ds_read_b128 %1, %8 offset:1024\n\t"
        "ds_read_b128 %2, %8 offset:2048\n\t"
        "ds_read_b128 %3, %8 offset:3072\n\t"
        "ds_read_b128 %4, %8 offset:4096\n\t"
        "ds_read_b128 %5, %8 offset:5120\n\t"
        "ds_read_b128 %6, %8 offset:6144\n\t"
        "ds_read_b128 %7, %8 offset:7168\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3]), "=&v"(r[4]), "=&v"(r[5]), "=&v"(r[6]), "=&v"(r[7])
        : "v"(ad)
        : "memory");
    DutyBlock d;
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            d.e[2 * h][q] = r[2 * q + h].x;
            d.e[2 * h + 1][q] = r[2 * q + h].y;
        }
    return d;
}

__device__ __forceinline__ uint64_t read_lse_staging(const u32x4 *xlse, int lane)
{
    const uint32_t ad = lds_addr(xlse) + 8u * (uint32_t)lane;
    uint64_t v;
    __asm__ volatile("ds_read_b64 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(v) : "v"(ad) : "memory");
    return v;
}

// Direct-to-LDS loads bypass the non-coherent cache levels like the atomic loads of the retry paths do.
constexpr int kDeviceScope = 16;          // the sc1 bit of the cache-policy operand

// 64 x 16 bytes: the 16-byte pairs 0 .. 63 of a row of 8-byte entries (row 16-byte aligned) that
// holds `pairs` pairs; lanes beyond the row repeat its last pair.
__device__ __forceinline__ void stage_entries(u32x4 *dst, const uint64_t *row, int pairs, int lane)
{
    const uint64_t *p = row + 2 * min(lane, pairs - 1);
    __builtin_amdgcn_global_load_lds(SP_GPTR(p), SP_LPTR(dst), 16, 0, kDeviceScope);
}

// The partials of rows row0 .. row0+3 of one exchange slot from every workgroup: eight loads.
__device__ __forceinline__ void stage_duty_block(u32x4 *xduty, const uint64_t *slot_base, int rows_pad, int n_wg,
                                                 int row0, int lane)
{
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint64_t *p = slot_base + (size_t)min(lane + 64 * q, n_wg - 1) * rows_pad + row0 + 2 * h;
            __builtin_amdgcn_global_load_lds(SP_GPTR(p), SP_LPTR(xduty + (2 * q + h) * 64), 16, 0, kDeviceScope);
        }
}

// A partial is ready when it carries the parity of this use of its slot and a non-zero sum.
// Entries beyond the last workgroup do not exist, rows outside the mask are padding: both count as ready.
__device__ __forceinline__ bool duty_ready(const DutyBlock &d, uint32_t par, int lane, int n_wg, uint32_t row_mask)
{
    uint32_t ok = 1u;           // branch-free: one straight-line test of the sixteen entries
#pragma unroll
    for (int r = 0; r < kDutyRows; ++r)
#pragma unroll
        for (int q = 0; q < 4; ++q)
            ok &= (uint32_t)(lane + 64 * q >= n_wg) | (((row_mask >> r) & 1u) ^ 1u) |
                  ((uint32_t)((uint32_t)(d.e[r][q] >> 63) == par) & (uint32_t)(((d.e[r][q] >> 32) & 0x7fffffffu) != 0));
    return ok != 0;
}

// Block of kDutyRows rows of phase p that workgroup w combines (>= rows_pad / kDutyRows: none).
// Blocks rotate over the workgroups.
__device__ __forceinline__ int duty_block_of(const FusedArgs &a, int p, int w)
{
    const int first = (int)(((uint32_t)p * (uint32_t)(a.rows_pad / kDutyRows)) % (uint32_t)a.n_wg);
    const int r = w - first;
    return r < 0 ? r + a.n_wg : r;
}

struct Shared {
    u32x4 *kring;                         // [8 waves][3 slots][32 rows x 8 chunks]
    u32x4 *q1[2], *q2[2];                 // Q tiles of the statistics / probability pass, by phase parity
    float2 (*wstats)[kFWaves][kMaxRowsF]; // [2]
    float (*cinit)[kMaxRowsF];            // [2]
    u32x4 *xduty, *xlse;
    int *fail;
};

// One step `s` of the software pipeline: everything between two workgroup barriers. Per wave, in
// program order (phase numbers in brackets are skipped when out of range):
//   mid     publish this workgroup's partials of eight rows of phase s-1 (all waves); the duty wave
//           requests the partials of its duty row of phase s-2; every wave requests its slices of
//           Q(s+1) for the next statistics pass and of Q(s-3) for the next probability pass
//   prob    probability pass of phase s-4 from ring slot s%4; loads of sub-tile 0 of K(s+1)
//   lse     the normaliser wave requests the normalisers of phase s-3
//   lift    wait for sub-tile 1 of K(s); lift K(s) into ring slot s%4
//   stats   statistics pass of phase s; loads of sub-tile 1 of K(s+1)
//   pre     wait for the Q slices (and the exchange data); duty wave: combine the duty row of phase
//           s-2 and publish its normaliser; normaliser wave: seeds of the probability pass of phase s-3
//   barrier
// Vector-memory operations per wave and step, oldest first: [publish store] [2 duty loads] Q, Q,
// 4 K loads (prob), [normaliser load], 4 K loads (stats); the bracketed ones exist on some waves or
// in some steps only, so every wait counts only operations that are certainly issued behind the
// ones it needs.
template <int NB, int GB, int SLOT, int PAR>
__device__ __forceinline__ void step(const FusedArgs &a, const LayerPtrs &kp, int s, int n_phases, Ring &ring,
                                     Acc<NB> &acc, const Shared &sh, int n_valid)
{
    // Lane-derived LDS and global offsets are recomputed every step instead of being kept in
    // registers across the whole loop (the opaque copy stops the compiler from hoisting them).
    int tid = threadIdx.x;
    __asm__ volatile("" : "+v"(tid));
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, hf = lane >> 5, col = lane & 31;
    const int w = blockIdx.x;
    const int pp = s - 1;                 // phase whose partials are published
    const int pc = s - 1 - kLag;          // phase of this step's probability pass
    const int pd = s - 2;                 // phase whose duty row is combined in this step
    const int pl = s - kLag;              // phase whose normalisers are fetched in this step
    const bool do_stats = s < n_phases, do_prob = pc >= 0 && pc < n_phases;

    // ---- mid ----
    if (wave == kPubWave) {
        if (pp >= 0 && pp < n_phases) {
            // one wave combines the eight per-wave statistics of every row (lane = row), maximum first,
            // then one exponential per source, and publishes the rows with one contiguous store
            float pm[kFWaves], pl8[kFWaves];
            {
                typedef __attribute__((ext_vector_type(2))) float f32x2;
                const uint32_t ad = lds_addr(&sh.wstats[1 - PAR][0][lane]);
                f32x2 r[kFWaves];
                static_assert(kFWaves == 8 && sizeof(float2) * kMaxRowsF == 512, "layout of the asm block");
                __asm__ volatile(
                    "ds_read_b64 %0, %8\n\t"
                    "ds_read_b64 %1, %8 offset:512\n\t"
                    "ds_read_b64 %2, %8 offset:1024\n\t"
                    "ds_read_b64 %3, %8 offset:1536\n\t"
                    "ds_read_b64 %4, %8 offset:2048\n\t"
                    "ds_read_b64 %5, %8 offset:2560\n\t"
                    "ds_read_b64 %6, %8 offset:3072\n\t"
                    "ds_read_b64 %7, %8 offset:3584\n\t"
                    "s_waitcnt lgkmcnt(0)"
                    : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3]), "=&v"(r[4]), "=&v"(r[5]), "=&v"(r[6]), "=&v"(r[7])
                    : "v"(ad)
                    : "memory");
#pragma unroll
                for (int i = 0; i < kFWaves; ++i) { pm[i] = r[i].x; pl8[i] = r[i].y; }
            }
            float m = pm[0];
#pragma unroll
            for (int i = 1; i < kFWaves; ++i) m = fmaxf(m, pm[i]);
            float l = 0.f;
#pragma unroll
            for (int i = 0; i < kFWaves; ++i) l += pl8[i] * fast_exp2((pm[i] - m) * a.c);
            if (lane < a.rows_pad) {
                const uint64_t bits = (uint64_t)__float_as_uint(m) | ((uint64_t)__float_as_uint(l) << 32) |
                                      ((uint64_t)((pp / kSlots) & 1) << 63);
                st64(a.part + ((size_t)(pp % kSlots) * a.n_wg + w) * a.rows_pad + lane, bits);
            }
        }
    } else if (wave == kDutyWave) {
        if (pd >= 0 && pd < n_phases) {
            const int blk = duty_block_of(a, pd, w);
            if (blk < a.rows_pad / kDutyRows)
                stage_duty_block(sh.xduty, a.part + (size_t)(pd % kSlots) * a.n_wg * a.rows_pad, a.rows_pad, a.n_wg,
                                 blk * kDutyRows, lane);
        }
    }
    {
        const PhaseId id1 = phase_of(min(s + 1, n_phases - 1), a.n_kv_heads);
        issue_q_slice<NB>(sh.q1[1 - PAR], a, id1.layer, id1.kv, wave, lane);
        const PhaseId id2 = phase_of(clampi(pl, 0, n_phases - 1), a.n_kv_heads);
        issue_q_slice<NB>(sh.q2[PAR], a, id2.layer, id2.kv, wave, lane);
    }

    // ---- probability pass of phase pc; sub-tile 0 of K(s+1) ----
    {
        const KIssue ki = k_issue_setup(a, kp, sh.kring, s + 1, 0, n_phases, n_valid, wave, lane);
        if (do_prob) {
            prob_pass<NB, GB>(ring.kf[SLOT], sh.q2[1 - PAR], sh.cinit[1 - PAR], acc, hf, col, ki);
            const PhaseId idc = phase_of(pc, a.n_kv_heads);
            if (idc.kv == a.n_kv_heads - 1 && (a.layer_agg == SP_LAYER_MEAN || idc.layer == a.n_layers - 1))
                close_layer<NB>(acc, a.c);
        } else {
            k_issue<kSubInstr>(ki, 0);
        }
    }
    if (wave == kLseWave) {
        const int pn = clampi(pl, 0, n_phases - 1);
        stage_entries(sh.xlse, a.lse + (size_t)(pn % kSlots) * a.rows_pad, a.rows_pad / 2, lane);
    }

    // ---- lift K(s), statistics pass of phase s; sub-tile 1 of K(s+1) ----
    vm_wait<2 + kSubInstr>();             // behind sub-tile 1 of K(s): at least Q, Q and the 4 loads of the prob part
    {
        const KIssue ki = k_issue_setup(a, kp, sh.kring, s + 1, 1, n_phases, n_valid, wave, lane);
        if (do_stats) {
#pragma unroll
            for (int s2 = 0; s2 < kNS; ++s2) lift_block(sub_slot(sh.kring, wave, s, s2), col, hf, ring.kf[SLOT][s2]);
            stats_pass<NB * GB>(a.c, ring.kf[SLOT], sh.q1[PAR], sh.wstats[PAR][wave], n_valid, wave, hf, col, ki);
        } else {
            k_issue<kSubInstr>(ki, 0);
        }
    }

    // ---- pre-barrier: exchange data in, seeds out ----
    if (wave == kLseWave) vm_wait<kSubInstr>(); else vm_wait<2 * kSubInstr>();
    if (wave == kDutyWave) {
        if (pd >= 0 && pd < n_phases) {
            const int blk = duty_block_of(a, pd, w);
            uint32_t row_mask = 0;
            if (blk < a.rows_pad / kDutyRows) {
#pragma unroll
                for (int r = 0; r < kDutyRows; ++r) {
                    int g, n;
                    if (row_valid<NB>(a, blk * kDutyRows + r, g, n)) row_mask |= 1u << r;
                }
            }
            if (row_mask != 0) {
                const uint32_t par = (uint32_t)(pd / kSlots) & 1u;
                const uint64_t *src = a.part + (size_t)(pd % kSlots) * a.n_wg * a.rows_pad + blk * kDutyRows;
                // fast path: the partials requested at the start of this step are all there; otherwise poll (bounded)
                DutyBlock de = read_duty_staging(sh.xduty, lane);
                if (__any(!duty_ready(de, par, lane, a.n_wg, row_mask)) && *sh.fail == 0) {
                    unsigned spins = 0;
                    do {
                        if (++spins > kSpinMax) { *sh.fail = 1; break; }
#pragma unroll
                        for (int r = 0; r < kDutyRows; ++r)
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                de.e[r][q] = ld64(src + (size_t)min(lane + 64 * q, a.n_wg - 1) * a.rows_pad + r);
                    } while (__any(!duty_ready(de, par, lane, a.n_wg, row_mask)));
                }
                // per row: maximum first, then one exponential per partial (short dependency chains, fixed order)
                float mine = 0.f;       // lane r keeps the normaliser of row r of the block
#pragma unroll
                for (int r = 0; r < kDutyRows; ++r) {
                    float pm[4], pl4[4], m = neg_inf();
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const bool valid = lane + 64 * q < a.n_wg;
                        pm[q] = valid ? __uint_as_float((uint32_t)de.e[r][q]) : neg_inf();
                        pl4[q] = valid ? __uint_as_float((uint32_t)(de.e[r][q] >> 32) & 0x7fffffffu) : 0.f;
                        m = fmaxf(m, pm[q]);
                    }
                    m = wave_max(m);
                    float l = 0.f;
#pragma unroll
                    for (int q = 0; q < 4; ++q) l += pl4[q] * fast_exp2((pm[q] - m) * a.c);
                    l = wave_sum(l);
                    const float v = -(m + fast_log2(l) * a.inv_c);
                    if (lane == r) mine = v;
                }
                if (lane < kDutyRows && ((row_mask >> lane) & 1u))
                    st64(a.lse + (size_t)(pd % kSlots) * a.rows_pad + blk * kDutyRows + lane,
                         (uint64_t)__float_as_uint(mine) | ((uint64_t)(uint32_t)(pd + 1) << 32));
            }
        }
    } else if (wave == kLseWave) {
        if (pl >= 0 && pl < n_phases && lane < a.rows_pad) {
            int g, n;
            float v = neg_inf();
            if (row_valid<NB>(a, lane, g, n)) {
                const uint64_t *src = a.lse + (size_t)(pl % kSlots) * a.rows_pad + lane;
                uint64_t entry = read_lse_staging(sh.xlse, lane);
                if ((uint32_t)(entry >> 32) != (uint32_t)(pl + 1) && *sh.fail == 0) {
                    unsigned spins = 0;
                    do {
                        if (++spins > kSpinMax) { *sh.fail = 1; break; }
                        entry = ld64(src);
                    } while ((uint32_t)(entry >> 32) != (uint32_t)(pl + 1));
                }
                v = __uint_as_float((uint32_t)entry);
            }
            const int rho = lane & 31;
            lds_store_f32(sh.cinit[PAR] + (lane & ~31) + ((rho >> 2) & 1) * 16 + 4 * (rho >> 3) + (rho & 3), v);
        }
    }
    lds_barrier();
}

template <int NB, int GB>
__global__ __launch_bounds__(kFThreads, 2) void sp_fused_kernel(FusedArgs a, LayerPtrs kp)
{
    __shared__ u32x4 kring[kFWaves * kSubSlots * kSubChunks];
    __shared__ u32x4 q1a[kMaxRowsF * kCH], q1b[kMaxRowsF * kCH], q2a[kMaxRowsF * kCH], q2b[kMaxRowsF * kCH];
    __shared__ float2 wstats[2][kFWaves][kMaxRowsF];
    __shared__ float cinit[2][kMaxRowsF];
    __shared__ u32x4 xduty[8 * 64];          // partials of the duty rows: 4 rows x 256 workgroups
    __shared__ u32x4 xlse[64];               // normaliser entries of one phase (64 used, the load moves 128)
    __shared__ int s_fail;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, hf = lane >> 5, col = lane & 31;
    const int w = blockIdx.x;
    const int n_phases = a.n_layers * a.n_kv_heads;
    const int64_t j0 = (int64_t)w * kFTile;
    const int n_valid = (int)((a.L - j0 < kFTile) ? a.L - j0 : kFTile);

    Shared sh;
    sh.kring = kring;
    sh.q1[0] = q1a; sh.q1[1] = q1b; sh.q2[0] = q2a; sh.q2[1] = q2b;
    sh.wstats = wstats; sh.cinit = cinit; sh.xduty = xduty; sh.xlse = xlse; sh.fail = &s_fail;

    if (tid < 2 * kMaxRowsF) cinit[tid / kMaxRowsF][tid % kMaxRowsF] = neg_inf();
    if (tid == 0) s_fail = 0;

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

    // prologue: this wave's slice of Q(0) and both sub-tiles of K(0); everything lands before step 0
    issue_q_slice<NB>(q1a, a, 0, 0, wave, lane);
#pragma unroll
    for (int s2 = 0; s2 < kNS; ++s2) {
        const KIssue ki = k_issue_setup(a, kp, kring, 0, s2, n_phases, n_valid, wave, lane);
        k_issue<kSubInstr>(ki, 0);
    }
    vm_wait<0>();
    lds_barrier();

    // The body is unrolled four times so that the fragment ring slot (s % 4) and the buffer parity
    // (s % 2) are compile-time; the trip count is rounded up, surplus steps do no work but keep the
    // instruction stream uniform. The last probability pass (phase n_phases - 1) runs in step n_phases + 3.
    const int n_steps = (n_phases + kLag + 1 + 3) / 4 * 4;
    for (int s0 = 0; s0 < n_steps; s0 += 4) {
        step<NB, GB, 0, 0>(a, kp, s0 + 0, n_phases, ring, acc, sh, n_valid);
        step<NB, GB, 1, 1>(a, kp, s0 + 1, n_phases, ring, acc, sh, n_valid);
        step<NB, GB, 2, 0>(a, kp, s0 + 2, n_phases, ring, acc, sh, n_valid);
        step<NB, GB, 3, 1>(a, kp, s0 + 3, n_phases, ring, acc, sh, n_valid);
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

size_t workspace_bytes(int rows_pad, int n_wg)
{
    return sp::align_up(sizeof(uint64_t) * ((size_t)kSlots * rows_pad * n_wg + (size_t)kSlots * rows_pad + 32), 256);
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

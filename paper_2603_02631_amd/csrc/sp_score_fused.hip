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
//  * one wave of some workgroup (rotating "duty") combines the partials of four
//    consecutive rows over all workgroups in a fixed order and publishes their
//    normalisers;
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
// A wait that gives up makes the whole call fail: the workgroup raises the
// call's status word at once, a duty that could not be completed publishes a
// poison entry that fails every workgroup reading it, and every workgroup
// reads the status word before it stores its scores (once any workgroup has
// passed that point all exchanged data is out, so none can fail after it).
//
// Variants of the same loop: head_dim 128 (256 keys per workgroup, a wave's two
// sub-tiles are the two halves of its 32 keys' rows: see the kernel's template
// flag W), paged keys and lookahead keys in the normaliser (flag EXTRA), and
// launches that carry several prompts of a ragged batch (a table of prompts,
// also under EXTRA: each prompt has its own workgroups, duty blocks and row of
// normalisers).
#include "sp_score_fused.hpp"

#include <atomic>
#include <cstring>

namespace {

using namespace sp_dev;
using sp_fused::FusedArgs;
using sp_fused::GroupTable;

constexpr int kD = 64;
constexpr int kKS = kD / 16;              // MFMA k-steps per row
constexpr int kFWaves = 8;
constexpr int kFThreads = kFWaves * 64;
constexpr int kNS = 2;                    // 32-key sub-tiles per wave
constexpr int kFTile = sp_fused::kTileKeys;   // 512 keys per workgroup per phase
constexpr int kSubInstr = 4;              // tile-load instructions per sub-tile (8 rows, 1 KB each)
constexpr int kSubSlots = 3;              // sub-tile slots in a wave's transit ring
constexpr int kLag = 3;                   // phases between statistics and probability pass
constexpr int kRing = kLag + 1;           // fragment ring: four phases
constexpr int kSlots = sp_fused::kSlots;  // exchange ring depth
constexpr int kMaxRowsF = sp_fused::kMaxRows;   // 64 padded query rows per kv head
constexpr int kPubWave = 0;                // the wave that publishes this workgroup's partials
constexpr int kDutyWave = 1;               // the wave that combines this workgroup's duty rows
constexpr int kDutyRows = 4;               // consecutive query rows one duty covers (32 bytes per source workgroup)
constexpr int kLseWave = 2;                // the wave that fetches the normalisers
constexpr uint32_t kPoisonTag = 0xffffffffu;   // normaliser entry of a duty that gave up

// LDS map in bytes. Everything but the K transit ring sits below 64 KB, so that reads of it can
// carry the buffer's place in the instruction's offset field.
constexpr int kQTileBytes = kMaxRowsF * kD * 2;                    // one Q tile: 64 rows x 128 bytes
constexpr int kWideHalf = 4096;                                    // head_dim 128: dims 64..127 of a Q tile's 32 rows sit here
constexpr int kOffQ1 = 0;                                          // [2] Q of the statistics pass, by phase parity
constexpr int kOffQ2 = kOffQ1 + 2 * kQTileBytes;                   // [2] Q of the probability pass
constexpr int kWstatsBytes = kFWaves * kMaxRowsF * 8;              // (max, sum) of 64 rows from 8 waves
constexpr int kOffWstats = kOffQ2 + 2 * kQTileBytes;               // [2]
constexpr int kOffCinit = kOffWstats + 2 * kWstatsBytes;           // [2][64] accumulator seeds
constexpr int kOffXduty = kOffCinit + 2 * kMaxRowsF * 4;           // 8 KB: partials of the duty rows
constexpr int kOffXlse = kOffXduty + 8192;                         // 1 KB: normaliser entries of one phase
constexpr int kOffXlook = kOffXlse + 1024;                         // 1 KB: lookahead-key terms of one phase's rows
constexpr int kOffFail = kOffXlook + 1024;
constexpr int kOffKring = (kOffFail + 16 + 1023) / 1024 * 1024;    // [8 waves][3 slots][32 rows x 128 bytes]
constexpr int kSubBytes = 32 * kD * 2;
constexpr int kLdsBytes = kOffKring + kFWaves * kSubSlots * kSubBytes;
static_assert(kOffKring < 65536, "offset fields hold 16 bits");

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

// Values that depend on the lane only, computed once: they cost a few registers and save the
// address arithmetic of every load and lift.
struct LaneConst {
    uint32_t ld[kKS];       // LDS byte address of this lane's fragment chunk t in a tile at LDS offset 0
    uint32_t ld8[kKS];      // the same in a sub-tile of 8-bit keys (rows of 64 bytes, 8 bytes per chunk)
    uint32_t koff[2];       // byte offset of this lane's chunk in an even / odd tile-load instruction (full tiles)
    int32_t qoff;           // byte offset of this lane's chunk of its wave's Q slice in a (layer, kv head) block; < 0: padding
};

// All LDS traffic of the main loop is written as asm: the compiler cannot tell which in-flight
// direct-to-LDS load targets which buffer and would put a full vector-memory wait in front of
// LDS accesses it can see. The kernel waits (vm_wait, barrier) for exactly what it is about to read.
__device__ __forceinline__ uint32_t lds_addr(const void *p) { return (uint32_t)reinterpret_cast<uintptr_t>(SP_LPTR(p)); }

// Direct-to-LDS loads of 64 lanes x 16 bytes into LDS bytes [lds_dst, lds_dst + 1024); lds_dst is
// uniform and travels in M0, which nothing else in this kernel uses. They are asm for the same
// reason, and so that the scalar-base form is used: a uniform 64-bit base plus a 32-bit lane offset.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ uint32_t uniform32(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
// The LDS destination is lds_base + LDS_IMM: call sites that differ only in the constant share one
// scalar register for the base.
template <int LDS_IMM>
__device__ __forceinline__ void dma_u(uint32_t lane_off, const void *base, uint32_t lds_base)
{
    const uint64_t b = reinterpret_cast<uintptr_t>(base);
    const uint64_t ub = (uint64_t)uniform32((uint32_t)b) | ((uint64_t)uniform32((uint32_t)(b >> 32)) << 32);
    __asm__ volatile("s_add_i32 m0, %2, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                     : : "v"(lane_off), "s"(ub), "s"(uniform32(lds_base)), "i"(LDS_IMM) : "memory", "m0", "scc");
}
// Per-lane addresses, bypassing the non-coherent cache levels like the atomic loads of the retry paths do.
__device__ __forceinline__ void dma_v_device(const void *addr, uint32_t lds_dst)
{
    __asm__ volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off sc1"
                     : : "v"(addr), "s"(uniform32(lds_dst)) : "memory", "m0");
}
#pragma clang diagnostic pop

// MFMA fragments of 32 rows of a swizzled 64-wide bf16 tile at compile-time LDS offset OFF:
// lane (col, hf) takes row col, 16-byte chunks 2t + hf.
template <int OFF>
__device__ __forceinline__ void lift_at(const LaneConst &lc, bf16x8 (&f)[kKS])
{
    static_assert(kKS == 4 && OFF >= 0 && OFF < 65536, "layout of the asm block");
    u32x4 r[kKS];
    __asm__ volatile(
        "ds_read_b128 %0, %4 offset:%8\n\t"
        "ds_read_b128 %1, %5 offset:%8\n\t"
        "ds_read_b128 %2, %6 offset:%8\n\t"
        "ds_read_b128 %3, %7 offset:%8\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3])
        : "v"(lc.ld[0]), "v"(lc.ld[1]), "v"(lc.ld[2]), "v"(lc.ld[3]), "i"(OFF)
        : "memory");
#pragma unroll
    for (int t = 0; t < kKS; ++t) f[t] = __builtin_bit_cast(bf16x8, r[t]);
}
// Both 32-key sub-tiles of a K tile (run-time slot offsets) and one 32-row Q block (compile-time
// offset) in one round trip to LDS.
template <int QOFF>
__device__ __forceinline__ void lift_k_and_q(const LaneConst &lc, uint32_t koff0, uint32_t koff1,
                                             bf16x8 (&kf)[kNS][kKS], bf16x8 (&qf)[kKS])
{
    static_assert(kKS == 4 && kNS == 2 && QOFF >= 0 && QOFF < 65536, "layout of the asm block");
    u32x4 r[12];
    uint32_t a0[kKS], a1[kKS];
#pragma unroll
    for (int t = 0; t < kKS; ++t) { a0[t] = lc.ld[t] + koff0; a1[t] = lc.ld[t] + koff1; }
    __asm__ volatile(
        "ds_read_b128 %0, %12\n\t"
        "ds_read_b128 %1, %13\n\t"
        "ds_read_b128 %2, %14\n\t"
        "ds_read_b128 %3, %15\n\t"
        "ds_read_b128 %8, %20 offset:%24\n\t"
        "ds_read_b128 %9, %21 offset:%24\n\t"
        "ds_read_b128 %10, %22 offset:%24\n\t"
        "ds_read_b128 %11, %23 offset:%24\n\t"
        "ds_read_b128 %4, %16\n\t"
        "ds_read_b128 %5, %17\n\t"
        "ds_read_b128 %6, %18\n\t"
        "ds_read_b128 %7, %19\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3]), "=&v"(r[4]), "=&v"(r[5]), "=&v"(r[6]), "=&v"(r[7]),
          "=&v"(r[8]), "=&v"(r[9]), "=&v"(r[10]), "=&v"(r[11])
        : "v"(a0[0]), "v"(a0[1]), "v"(a0[2]), "v"(a0[3]), "v"(a1[0]), "v"(a1[1]), "v"(a1[2]), "v"(a1[3]),
          "v"(lc.ld[0]), "v"(lc.ld[1]), "v"(lc.ld[2]), "v"(lc.ld[3]), "i"(QOFF)
        : "memory");
#pragma unroll
    for (int t = 0; t < kKS; ++t) {
        kf[0][t] = __builtin_bit_cast(bf16x8, r[t]);
        kf[1][t] = __builtin_bit_cast(bf16x8, r[4 + t]);
        qf[t] = __builtin_bit_cast(bf16x8, r[8 + t]);
    }
}

// 8-bit keys: both 32-key sub-tiles of a K tile (rows of 64 codes; this lane's eight codes of k-step t
// are one 8-byte read) and one 32-row Q block in one round trip to LDS, the codes widened to bf16.
template <int QOFF>
__device__ __forceinline__ void lift_k8_and_q(const LaneConst &lc, uint32_t koff0, uint32_t koff1,
                                              bf16x8 (&kf)[kNS][kKS], bf16x8 (&qf)[kKS])
{
    static_assert(kKS == 4 && kNS == 2 && QOFF >= 0 && QOFF < 65536, "layout of the asm block");
    typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
    u32x2 r[8];
    u32x4 q[4];
    uint32_t a0[kKS], a1[kKS];
#pragma unroll
    for (int t = 0; t < kKS; ++t) { a0[t] = lc.ld8[t] + koff0; a1[t] = lc.ld8[t] + koff1; }
    __asm__ volatile(
        "ds_read_b64 %0, %12\n\t"
        "ds_read_b64 %1, %13\n\t"
        "ds_read_b64 %2, %14\n\t"
        "ds_read_b64 %3, %15\n\t"
        "ds_read_b128 %8, %20 offset:%24\n\t"
        "ds_read_b128 %9, %21 offset:%24\n\t"
        "ds_read_b128 %10, %22 offset:%24\n\t"
        "ds_read_b128 %11, %23 offset:%24\n\t"
        "ds_read_b64 %4, %16\n\t"
        "ds_read_b64 %5, %17\n\t"
        "ds_read_b64 %6, %18\n\t"
        "ds_read_b64 %7, %19\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3]), "=&v"(r[4]), "=&v"(r[5]), "=&v"(r[6]), "=&v"(r[7]),
          "=&v"(q[0]), "=&v"(q[1]), "=&v"(q[2]), "=&v"(q[3])
        : "v"(a0[0]), "v"(a0[1]), "v"(a0[2]), "v"(a0[3]), "v"(a1[0]), "v"(a1[1]), "v"(a1[2]), "v"(a1[3]),
          "v"(lc.ld[0]), "v"(lc.ld[1]), "v"(lc.ld[2]), "v"(lc.ld[3]), "i"(QOFF)
        : "memory");
#pragma unroll
    for (int t = 0; t < kKS; ++t) {
        kf[0][t] = __builtin_bit_cast(bf16x8, e4m3x8_to_bf16x8(r[t].x, r[t].y));
        kf[1][t] = __builtin_bit_cast(bf16x8, e4m3x8_to_bf16x8(r[4 + t].x, r[4 + t].y));
        qf[t] = __builtin_bit_cast(bf16x8, q[t]);
    }
}

// One 32-row Q block (compile-time offset) and the sixteen accumulator seeds at seed_ad (64-byte
// aligned) in one round trip to LDS.
template <int QOFF>
__device__ __forceinline__ void lift_q_and_seed(const LaneConst &lc, uint32_t seed_ad, bf16x8 (&qf)[kKS], f32x16 &seed)
{
    static_assert(kKS == 4 && QOFF >= 0 && QOFF < 65536, "layout of the asm block");
    typedef __attribute__((ext_vector_type(4))) float f32x4;
    u32x4 r[kKS];
    f32x4 c[4];
    __asm__ volatile(
        "ds_read_b128 %0, %8 offset:%13\n\t"
        "ds_read_b128 %1, %9 offset:%13\n\t"
        "ds_read_b128 %2, %10 offset:%13\n\t"
        "ds_read_b128 %3, %11 offset:%13\n\t"
        "ds_read_b128 %4, %12\n\t"
        "ds_read_b128 %5, %12 offset:16\n\t"
        "ds_read_b128 %6, %12 offset:32\n\t"
        "ds_read_b128 %7, %12 offset:48\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3]), "=&v"(c[0]), "=&v"(c[1]), "=&v"(c[2]), "=&v"(c[3])
        : "v"(lc.ld[0]), "v"(lc.ld[1]), "v"(lc.ld[2]), "v"(lc.ld[3]), "v"(seed_ad), "i"(QOFF)
        : "memory");
#pragma unroll
    for (int t = 0; t < kKS; ++t) qf[t] = __builtin_bit_cast(bf16x8, r[t]);
#pragma unroll
    for (int v = 0; v < 4; ++v) { seed[4 * v] = c[v].x; seed[4 * v + 1] = c[v].y; seed[4 * v + 2] = c[v].z; seed[4 * v + 3] = c[v].w; }
}

__device__ __forceinline__ void lds_store_f32(uint32_t ad, float v)
{
    __asm__ volatile("ds_write_b32 %0, %1" : : "v"(ad), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_store_f2(uint32_t ad, float2 v)
{
    __asm__ volatile("ds_write_b64 %0, %1" : : "v"(ad), "v"(v) : "memory");
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

__device__ __forceinline__ float lane_value(float v, int lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}
__device__ __forceinline__ float wave_max(float v)
{
    v = fmaxf(v, dpp_move<kDppXor1>(v));
    v = fmaxf(v, dpp_move<kDppXor2>(v));
    v = fmaxf(v, dpp_move<kDppHalfMirror>(v));
    v = fmaxf(v, dpp_move<kDppMirror>(v));
    return fmaxf(fmaxf(lane_value(v, 0), lane_value(v, 16)), fmaxf(lane_value(v, 32), lane_value(v, 48)));
}
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_move<kDppXor1>(v);
    v += dpp_move<kDppXor2>(v);
    v += dpp_move<kDppHalfMirror>(v);
    v += dpp_move<kDppMirror>(v);
    return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}

// (layer, kv head) of a phase, walked step by step instead of divided out every time.
struct PhaseCtr { int layer, kv; };
__device__ __forceinline__ PhaseCtr phase_at(int p, int n_phases, int n_kv)
{
    p = clampi(p, 0, n_phases - 1);
    PhaseCtr r; r.layer = p / n_kv; r.kv = p - r.layer * n_kv; return r;
}
// c holds clamp(p_next - 1, 0, n_phases - 1); make it hold clamp(p_next, 0, n_phases - 1).
__device__ __forceinline__ void phase_advance(PhaseCtr &c, int p_next, int n_phases, int n_kv)
{
    if (p_next > 0 && p_next < n_phases) {
        if (++c.kv == n_kv) { c.kv = 0; ++c.layer; }
    }
}

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
// contiguous); a 32-key sub-tile takes four of them: a uniform base that steps by 8 keys, plus the
// lane's constant offset (even / odd instruction).
struct KIssue {
    uint32_t lds_dst;         // LDS byte address of the sub-tile slot being refilled (this wave's)
    const char *base;         // first key of the sub-tile in the (layer, kv head) being fetched (uniform)
    uint32_t step_bytes;      // bytes between the first keys of consecutive instructions (8 keys)
};

// Issues instructions first .. first+COUNT-1 of the sub-tile (first and COUNT compile-time at call sites).
template <int IDX>
__device__ __forceinline__ void k_issue_one(const KIssue &ki, const uint32_t (&voff)[2])
{
    dma_u<IDX * 1024>(voff[IDX & 1], ki.base + (uint32_t)IDX * ki.step_bytes, ki.lds_dst);
}
template <int COUNT>
__device__ __forceinline__ void k_issue(const KIssue &ki, const uint32_t (&voff)[2], int first)
{
    static_assert(kSubInstr == 4, "instruction indices 0..3");
#pragma unroll
    for (int i = 0; i < COUNT; ++i) {
        switch (first + i) {          // compile-time after unrolling
        case 0: k_issue_one<0>(ki, voff); break;
        case 1: k_issue_one<1>(ki, voff); break;
        case 2: k_issue_one<2>(ki, voff); break;
        default: k_issue_one<3>(ki, voff); break;
        }
    }
}

// Sub-tile s2 of phase p lives in slot (2p + s2) mod 3 of its wave's transit ring; slot0 = 2p mod 3.
__device__ __forceinline__ uint32_t sub_slot_off(int wave, int slot0, int s2)
{
    int slot = slot0 + s2;
    slot = slot >= kSubSlots ? slot - kSubSlots : slot;
    return (uint32_t)(kOffKring + (wave * kSubSlots + slot) * kSubBytes);
}

template <int NB>
struct Acc {
    float mx[kNS][NB][4];
    float total[kNS];
};

// ---- probability pass of one phase from the fragment ring; tile loads are issued between the MFMA steps ----
// Of the four loads of sub-tile 0 two are issued right after the barrier and two between the MFMA steps of
// the probability pass (8-bit keys: two loads a sub-tile, one and one).

// F8: logits are in units of the phase's key scale `ks`; a phase's head maximum is brought to common
// units before it meets other phases'. One tile load instead of two (half the bytes per sub-tile).
template <int NB, int GB, int PAR, bool W, bool F8>
__device__ __forceinline__ void prob_pass(const bf16x8 (&kf)[kNS][kKS], const LaneConst &lc, uint32_t cinit_ad,
                                          Acc<NB> &acc, const KIssue &ki, const uint32_t (&voff)[2], float ks)
{
    static_assert(NB * GB == 1 || NB * GB == 2, "one load per row block, or one per step");
    constexpr int kMid = F8 ? 1 : 2;
    if constexpr (W) {
        // head_dim 128: one chain of eight MFMA steps over both halves of the 32 keys' rows
        static_assert(NB == 1 && GB == 1, "one block of 32 query rows");
        bf16x8 q0[kKS], q1[kKS];
        f32x16 d;
        lift_q_and_seed<kOffQ2 + PAR * kQTileBytes>(lc, cinit_ad, q0, d);
        lift_at<kOffQ2 + PAR * kQTileBytes + kWideHalf>(lc, q1);
#pragma unroll
        for (int t = 0; t < kKS; ++t) d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q0[t], kf[0][t], d, 0, 0, 0);
        k_issue<1>(ki, voff, kMid);
#pragma unroll
        for (int t = 0; t < kKS; ++t) d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q1[t], kf[1][t], d, 0, 0, 0);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (F8) acc.mx[0][0][e] = fmaxf(acc.mx[0][0][e], fmaxf(max3(d[e], d[4 + e], d[8 + e]), d[12 + e]) * ks);
            else acc.mx[0][0][e] = max3(max3(d[e], d[4 + e], d[8 + e]), d[12 + e], acc.mx[0][0][e]);
        }
        if (!F8) k_issue<1>(ki, voff, kMid + 1);
        __builtin_amdgcn_sched_barrier(0);
        return;
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
        for (int gb = 0; gb < GB; ++gb) {
            const int blk = gb * NB + nb;
            bf16x8 qf[kKS];
            f32x16 ci;
            if (blk == 0) lift_q_and_seed<kOffQ2 + PAR * kQTileBytes>(lc, cinit_ad, qf, ci);
            else lift_q_and_seed<kOffQ2 + PAR * kQTileBytes + 4096>(lc, cinit_ad + 128, qf, ci);
#pragma unroll
            for (int s = 0; s < kNS; ++s) {
                f32x16 d = ci;
#pragma unroll
                for (int t = 0; t < kKS; ++t) d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[t], kf[s][t], d, 0, 0, 0);
                // d[r]: group head r/4, lookahead row 8*nb + 4*hf + r%4, key (wave*2+s)*32 + col
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (F8) acc.mx[s][nb][e] = fmaxf(acc.mx[s][nb][e], fmaxf(max3(d[e], d[4 + e], d[8 + e]), d[12 + e]) * ks);
                    else acc.mx[s][nb][e] = max3(max3(d[e], d[4 + e], d[8 + e]), d[12 + e], acc.mx[s][nb][e]);
                }
                if (F8) { if (blk == 0 && s == 0) k_issue<1>(ki, voff, kMid); }
                else if (NB * GB == 1) k_issue<1>(ki, voff, kMid + s);
                else if (s == kNS - 1) k_issue<1>(ki, voff, kMid + blk);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
}

template <int NB, int NSE>
__device__ __forceinline__ void close_layer(Acc<NB> &acc, float c)
{
#pragma unroll
    for (int s = 0; s < NSE; ++s) {
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

// 64 x 16 bytes: the 16-byte pairs 0 .. 63 of a row of 8-byte entries (row 16-byte aligned) that
// holds `pairs` pairs; lanes beyond the row repeat its last pair.
__device__ __forceinline__ void stage_entries(uint32_t lds_dst, const uint64_t *row, int pairs, int lane)
{
    dma_v_device(row + 2 * min(lane, pairs - 1), lds_dst);
}

// The normaliser wave's requests of one step: the rows' lookahead-key terms (when the call has
// them; 4-byte entries, four to a lane) and, behind them, the normaliser entries. Loads return in
// order, so the wait for the normalisers covers both.
__device__ __forceinline__ void stage_exchange_rows(uint32_t xlse_ad, const uint64_t *lse_row, const float *look_row,
                                                    int rows_pad, int lane)
{
    if (look_row != nullptr) dma_v_device(look_row + 4 * min(lane, rows_pad / 4 - 1), xlse_ad + (kOffXlook - kOffXlse));
    stage_entries(xlse_ad, lse_row, rows_pad / 2, lane);
}

// ---- statistics pass of one phase: per-wave (max, sum exp) of every row into wstats ----
// Logits of 32 keys (one sub-tile) against 32 query rows: d[r] is key 8*(r/4) + 4*hf + r%4 of the
// sub-tile, query row col.
__device__ __forceinline__ f32x16 logits32(const bf16x8 (&kf)[kKS], const bf16x8 (&qf)[kKS])
{
    f32x16 d = {0.f};
#pragma unroll
    for (int t = 0; t < kKS; ++t) d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t], qf[t], d, 0, 0, 0);
    return d;
}

// Folds the 16 logits of a lane into its running (max, sum exp); only keys lo <= key < hi of the
// sub-tile are this workgroup's (all 32 except in the prompt's last tile).
__device__ __forceinline__ void fold_logits(const f32x16 &d, float &m, float &l, float c, int lo, int hi, int hf)
{
    if (lo <= 0 && hi >= 32) {
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
    } else if (lo < 32 && hi > 0) {
        float tm = neg_inf();
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = 8 * (r >> 2) + 4 * hf + (r & 3);
            if (key >= lo && key < hi) tm = fmaxf(tm, d[r]);
        }
        if (tm > neg_inf()) {
            const float mn = fmaxf(m, tm);
            l *= fast_exp2((m - mn) * c);
            m = mn;
            const float mc = mn * c;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = 8 * (r >> 2) + 4 * hf + (r & 3);
                if (key >= lo && key < hi) l += fast_exp2(fmaf(d[r], c, -mc));
            }
        }
    }
}

__device__ __forceinline__ void store_row_stats(uint32_t ad, float m, float l, float c, int hf)
{
    const float m2 = __shfl_xor(m, 32), l2 = __shfl_xor(l, 32);
    lse_merge(m, l, m2, l2, c);
    if (hf == 0) lds_store_f2(ad, make_float2(m, l));
}

// Lifts the K tile of the phase into kf, then runs the MFMA steps one ahead of the arithmetic on
// their results, so that the matrix pipe works under the exponentials of the previous step. One
// tile load is issued after each of the four steps (with one row block: two per step). On the
// normaliser wave (lse_row != nullptr) the request for the normalisers follows the first step: late
// enough for the duty workgroups' stores to be visible, early enough to land before the barrier.
template <int NBLK, bool F8>
constexpr int kLoadsBehindLse = F8 ? 1 : kSubInstr - kSubInstr / (NBLK * kNS);

template <int NBLK, int PAR, bool W, bool F8>
__device__ __forceinline__ void stats_pass(float c, bf16x8 (&kf)[kNS][kKS], const LaneConst &lc, uint32_t koff0,
                                           uint32_t koff1, uint32_t wstats_ad, int lo0, int hi0, int lane,
                                           const KIssue &ki, const uint32_t (&voff)[2], const uint64_t *lse_row,
                                           const float *look_row, int rows_pad, uint32_t xlse_ad)
{
    // tile-load instructions issued after each MFMA step (8-bit keys: two in all, after the first two steps)
    constexpr int kPerStep = F8 ? 1 : kSubInstr / (NBLK * kNS);
    constexpr int kLate = F8 ? 0 : kPerStep;             // after the third and fourth step
    const int hf = lane >> 5;
    if constexpr (W) {
        // head_dim 128: the two sub-tiles are the two halves of the rows of this wave's 32 keys
        static_assert(NBLK == 1, "one block of 32 query rows");
        bf16x8 q0[kKS], q1[kKS];
        if (F8) lift_k8_and_q<kOffQ1 + PAR * kQTileBytes>(lc, koff0, koff1, kf, q0);
        else lift_k_and_q<kOffQ1 + PAR * kQTileBytes>(lc, koff0, koff1, kf, q0);
        lift_at<kOffQ1 + PAR * kQTileBytes + kWideHalf>(lc, q1);
        f32x16 d = logits32(kf[0], q0);
#pragma unroll
        for (int t = 0; t < kKS; ++t) d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[1][t], q1[t], d, 0, 0, 0);
        k_issue<kPerStep>(ki, voff, 0);
        if (lse_row != nullptr) stage_exchange_rows(xlse_ad, lse_row, look_row, rows_pad, lane);
        __builtin_amdgcn_sched_barrier(0);
        float m = neg_inf(), l = 0.f;
        fold_logits(d, m, l, c, lo0, hi0, hf);
        store_row_stats(wstats_ad, m, l, c, hf);
        k_issue<kPerStep>(ki, voff, kPerStep);
        __builtin_amdgcn_sched_barrier(0);
        return;
    }
    const int lo1 = lo0 - 32, hi1 = hi0 - 32;      // this wave's keys lo0 <= key < hi0 (of 64) are the workgroup's
    bf16x8 qf[kKS];
    if (F8) lift_k8_and_q<kOffQ1 + PAR * kQTileBytes>(lc, koff0, koff1, kf, qf);
    else lift_k_and_q<kOffQ1 + PAR * kQTileBytes>(lc, koff0, koff1, kf, qf);
    f32x16 da = logits32(kf[0], qf);
    f32x16 db = logits32(kf[1], qf);
    float m = neg_inf(), l = 0.f;
    fold_logits(da, m, l, c, lo0, hi0, hf);
    k_issue<kPerStep>(ki, voff, 0);
    if (lse_row != nullptr) stage_exchange_rows(xlse_ad, lse_row, look_row, rows_pad, lane);
    __builtin_amdgcn_sched_barrier(0);
    if (NBLK == 2) {
        lift_at<kOffQ1 + PAR * kQTileBytes + 4096>(lc, qf);
        da = logits32(kf[0], qf);
    }
    fold_logits(db, m, l, c, lo1, hi1, hf);
    store_row_stats(wstats_ad, m, l, c, hf);
    k_issue<kPerStep>(ki, voff, kPerStep);
    __builtin_amdgcn_sched_barrier(0);
    if (NBLK == 2) {
        db = logits32(kf[1], qf);
        m = neg_inf(); l = 0.f;
        fold_logits(da, m, l, c, lo0, hi0, hf);
        k_issue<kLate>(ki, voff, 2 * kPerStep);
        __builtin_amdgcn_sched_barrier(0);
        fold_logits(db, m, l, c, lo1, hi1, hf);
        store_row_stats(wstats_ad + 256, m, l, c, hf);
        k_issue<kLate>(ki, voff, 3 * kPerStep);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Exchange data requested with direct-to-LDS loads lands in two small staging areas, each private
// to one wave. Partials are stored workgroup-major, part[slot][workgroup][row], so that a workgroup
// publishes all its rows with one contiguous store; a duty covers kDutyRows consecutive rows, i.e.
// one 32-byte piece of every workgroup's line. xduty receives them as 16-byte pairs of rows:
// chunk (2q + h) * 64 + lane holds rows 2h and 2h+1 of the block from workgroup lane + 64q.
struct DutyBlock { uint64_t e[kDutyRows][4]; };     // [row of the block][workgroup lane + 64q]

__device__ __forceinline__ DutyBlock read_duty_staging(uint32_t lds0, int lane)
{
    static_assert(kDutyRows == 4, "layout of the asm block");
    typedef __attribute__((ext_vector_type(2))) uint64_t u64x2;
    const uint32_t ad = lds0 + kOffXduty + 16u * (uint32_t)lane;
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

__device__ __forceinline__ uint64_t read_lse_staging(uint32_t lds0, int lane)
{
    const uint32_t ad = lds0 + kOffXlse + 8u * (uint32_t)lane;
    uint64_t v;
    __asm__ volatile("ds_read_b64 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(v) : "v"(ad) : "memory");
    return v;
}

__device__ __forceinline__ float read_look_staging(uint32_t lds0, int lane)
{
    const uint32_t ad = lds0 + kOffXlook + 4u * (uint32_t)lane;
    float v;
    __asm__ volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(v) : "v"(ad) : "memory");
    return v;
}

// The partials of rows row0 .. row0+3 of one exchange slot from every workgroup: eight loads.
__device__ __forceinline__ void stage_duty_block(uint32_t xduty, const uint64_t *slot_base, int rows_pad, int n_wg,
                                                 int row0, int lane)
{
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int h = 0; h < 2; ++h)
            dma_v_device(slot_base + (size_t)min(lane + 64 * q, n_wg - 1) * rows_pad + row0 + 2 * h,
                         xduty + (2 * q + h) * 1024);
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

// A wait gave up (or met a poison entry): the workgroup stops waiting for anything and the call's
// status word is raised at once, so that every workgroup finds it before storing its scores.
__device__ __forceinline__ void raise_failure(const FusedArgs &a, int *fail)
{
    *fail = 1;
    __hip_atomic_store(a.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Uniform state that walks along with the steps.
struct Walk {
    PhaseCtr k;       // phase s + 1: next statistics pass (its K tile is being fetched)
    const char *kptr; // this wave's first key of that phase
    PhaseCtr c;       // phase s - 4: this step's probability pass
    int slot0;        // transit slot of sub-tile 0 of phase s: 2s mod 3
    int dfirst;       // workgroup that combines block 0 of phase s - 2; blocks rotate over the workgroups
};

// One step `s` of the software pipeline: everything between two workgroup barriers. Per wave, in
// program order (phase numbers in brackets are skipped when out of range):
//   mid     one wave publishes this workgroup's partials of phase s-1; the duty wave requests the
//           partials of its duty rows of phase s-2; every wave requests its slices of Q(s+1) for
//           the next statistics pass and of Q(s-3) for the next probability pass
//   prob    probability pass of phase s-4 from ring slot s%4; loads of sub-tile 0 of K(s+1)
//   lift    wait for sub-tile 1 of K(s); lift K(s) into ring slot s%4
//   stats   statistics pass of phase s; loads of sub-tile 1 of K(s+1); after its first step the
//           normaliser wave requests the normalisers of phase s-3
//   pre     wait for the Q slices (and the exchange data); duty wave: combine the duty rows of phase
//           s-2 and publish their normalisers; normaliser wave: seeds of the probability pass of phase s-3
//   barrier
// Vector-memory operations per wave and step, oldest first: [publish store] [8 duty loads] [Q] [Q]
// 4 K loads (prob), [normaliser load], 4 K loads (stats); the bracketed ones exist on some waves or
// in some steps only, so every wait counts only operations that are certainly issued behind the
// ones it needs.
// EXTRA selects the variant that also serves paged keys (an upper bound on the tile's rows) and
// lookahead keys in the normaliser; the plain variant carries none of their code or registers.
template <int NB, int GB, int SLOT, int PAR, bool EXTRA, bool W, bool F8>
__device__ __forceinline__ void step(const FusedArgs &a, const LayerPtrs &kp, const GroupTable &gt, int s, int n_phases, Ring &ring,
                                     Acc<NB> &acc, const LaneConst &lc, Walk &wk, unsigned char *lds, uint32_t lds0,
                                     uint64_t wave_off, int r_range)
{
    // Other lane-derived values are recomputed every step instead of being kept in registers across
    // the whole loop (the opaque copy stops the compiler from hoisting them).
    int tid = threadIdx.x;
    __asm__ volatile("" : "+v"(tid));
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int w = blockIdx.x;
    const int pp = s - 1;                 // phase whose partials are published
    const int pc = s - 1 - kLag;          // phase of this step's probability pass
    const int pd = s - 2;                 // phase whose duty rows are combined in this step
    const int pl = s - kLag;              // phase whose normalisers are fetched in this step
    const bool do_stats = s < n_phases, do_prob = pc >= 0 && pc < n_phases;
    constexpr int kSI = F8 ? kSubInstr / 2 : kSubInstr;     // tile-load instructions per sub-tile
    constexpr int kMid = F8 ? 1 : 2;                        // of them, for sub-tile 0: issued right after the barrier
    constexpr uint32_t kElem = F8 ? 1u : 2u;                // bytes per key element
    const uint32_t stride_bytes = (uint32_t)a.k_stride_token * kElem;
    // 8-bit keys: the exponent's scale of a phase is c times that phase's key scale
    const float c_stats = F8 ? a.c * a.kscale[clampi(s, 0, n_phases - 1)] : a.c;
    const float c_pub = F8 ? a.c * a.kscale[clampi(pp, 0, n_phases - 1)] : a.c;
    const float c_duty = F8 ? a.c * a.kscale[clampi(pd, 0, n_phases - 1)] : a.c;
    const float ks_prob = F8 ? a.kscale[clampi(pc, 0, n_phases - 1)] : 1.f;
    // Duty blocks of a phase: kDutyRows consecutive rows of one prompt (launches over several prompts have
    // blocks_per_prompt of them for each); block i goes to workgroup dfirst + i. src_w0 / src_n: the
    // workgroups whose partials the block combines (its prompt's), lse_idx: the prompt's row of normalisers.
    const int blocks_per_prompt = a.rows_pad / kDutyRows;
    int duty_blk = wk.dfirst <= w ? w - wk.dfirst : w - wk.dfirst + a.n_wg;
    if (pd < 0 || pd >= n_phases || duty_blk >= blocks_per_prompt * a.n_gp) duty_blk = -1;
    int src_w0 = 0, src_n = a.n_wg, lse_idx = 0;
    if (EXTRA && a.n_gp > 1 && duty_blk >= 0) {
        lse_idx = duty_blk / blocks_per_prompt;
        duty_blk -= lse_idx * blocks_per_prompt;
        src_w0 = gt.w0[lse_idx];
        src_n = gt.w0[lse_idx + 1] - src_w0;
    }

    // ---- mid ----
    if (wave == kPubWave) {
        if (pp >= 0 && pp < n_phases) {
            // one wave combines the eight per-wave statistics of every row (lane = row), maximum first,
            // then one exponential per source, and publishes the rows with one contiguous store
            float pm[kFWaves], pl8[kFWaves];
            {
                typedef __attribute__((ext_vector_type(2))) float f32x2;
                const uint32_t ad = lds0 + 8u * (uint32_t)lane;
                f32x2 r[kFWaves];
                static_assert(kFWaves == 8 && kMaxRowsF * 8 == 512, "layout of the asm block");
                __asm__ volatile(
                    "ds_read_b64 %0, %8 offset:%9\n\t"
                    "ds_read_b64 %1, %8 offset:%9+512\n\t"
                    "ds_read_b64 %2, %8 offset:%9+1024\n\t"
                    "ds_read_b64 %3, %8 offset:%9+1536\n\t"
                    "ds_read_b64 %4, %8 offset:%9+2048\n\t"
                    "ds_read_b64 %5, %8 offset:%9+2560\n\t"
                    "ds_read_b64 %6, %8 offset:%9+3072\n\t"
                    "ds_read_b64 %7, %8 offset:%9+3584\n\t"
                    "s_waitcnt lgkmcnt(0)"
                    : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3]), "=&v"(r[4]), "=&v"(r[5]), "=&v"(r[6]), "=&v"(r[7])
                    : "v"(ad), "i"(kOffWstats + (1 - PAR) * kWstatsBytes)
                    : "memory");
#pragma unroll
                for (int i = 0; i < kFWaves; ++i) { pm[i] = r[i].x; pl8[i] = r[i].y; }
            }
            float m = pm[0];
#pragma unroll
            for (int i = 1; i < kFWaves; ++i) m = fmaxf(m, pm[i]);
            float l = 0.f;
#pragma unroll
            for (int i = 0; i < kFWaves; ++i) l += pl8[i] * fast_exp2((pm[i] - m) * c_pub);
            if (lane < a.rows_pad) {
                const uint64_t bits = (uint64_t)__float_as_uint(m) | ((uint64_t)__float_as_uint(l) << 32) |
                                      ((uint64_t)((pp / kSlots) & 1) << 63);
                st64(a.part + ((size_t)(pp % kSlots) * a.n_wg + w) * a.rows_pad + lane, bits);
            }
        }
    } else if (wave == kDutyWave) {
        if (duty_blk >= 0)
            stage_duty_block(lds0 + kOffXduty, a.part + ((size_t)(pd % kSlots) * a.n_wg + src_w0) * a.rows_pad, a.rows_pad,
                             src_n, duty_blk * kDutyRows, lane);
    }
    const char *kbase = wk.kptr;
    int slot_next = wk.slot0 + 2;         // sub-tile 0 of phase s + 1
    slot_next = slot_next >= kSubSlots ? slot_next - kSubSlots : slot_next;
    // past the last phase the loads shrink to one 16-byte piece per instruction: the count stays fixed
    const uint32_t live = s + 1 < n_phases ? 0xffffffffu : 0u;
    const uint32_t voff[2] = {lc.koff[0] & live, lc.koff[1] & live};
    KIssue ki;
    ki.lds_dst = lds0 + sub_slot_off(wave, slot_next, 0);
    ki.base = kbase;
    ki.step_bytes = (F8 ? 16u : 8u) * stride_bytes;
    if (lc.qoff >= 0) {       // padding rows of the Q tiles stay zero; the Q blocks of consecutive phases are contiguous
        const uint32_t qblock = (uint32_t)(a.group * a.n_q * kD * 2) * (W ? 2u : 1u);
        const char *q1src = reinterpret_cast<const char *>(a.q) + (uint32_t)min(s + 1, n_phases - 1) * qblock;
        const char *q2src = reinterpret_cast<const char *>(a.q) + (uint32_t)clampi(pl, 0, n_phases - 1) * qblock;
        dma_u<kOffQ1 + (1 - PAR) * kQTileBytes>((uint32_t)lc.qoff, q1src, lds0 + wave * 1024);
        dma_u<kOffQ2 + PAR * kQTileBytes>((uint32_t)lc.qoff, q2src, lds0 + wave * 1024);
    }
    k_issue<kMid>(ki, voff, 0);

    // ---- probability pass of phase pc; sub-tile 0 of K(s+1) ----
    {
        if (do_prob) {
            const uint32_t cinit_ad = lds0 + kOffCinit + (1 - PAR) * (kMaxRowsF * 4) + ((uint32_t)(lane & 32) << 1);
            prob_pass<NB, GB, 1 - PAR, W, F8>(ring.kf[SLOT], lc, cinit_ad, acc, ki, voff, ks_prob);
            if (wk.c.kv == a.n_kv_heads - 1 && (a.layer_agg == SP_LAYER_MEAN || wk.c.layer == a.n_layers - 1))
                close_layer<NB, W ? 1 : kNS>(acc, a.c);
        } else {
            k_issue<kSI - kMid>(ki, voff, kMid);
        }
    }

    // ---- lift K(s), statistics pass of phase s; sub-tile 1 of K(s+1) ----
    vm_wait<kSI>();                       // behind sub-tile 1 of K(s): at least the loads of sub-tile 0 of K(s+1)
    {
        KIssue ki;
        ki.lds_dst = lds0 + sub_slot_off(wave, slot_next, 1);
        ki.base = kbase + (W ? (int64_t)(kD * kElem) : (int64_t)32 * stride_bytes);     // W: the rows' second halves
        ki.step_bytes = (F8 ? 16u : 8u) * stride_bytes;
        const uint64_t *lse_row = wave == kLseWave ? a.lse + ((size_t)(clampi(pl, 0, n_phases - 1) % kSlots) * a.n_gp + a.p_idx) * a.rows_pad : nullptr;
        const float *look_row = nullptr;
        if (EXTRA && a.look != nullptr) look_row = a.look + (size_t)clampi(pl, 0, n_phases - 1) * a.rows_pad;
        // r_range = r_lo | r_hi << 16 (r_hi = 512 without EXTRA): this wave's share of it
        constexpr int kWaveKeys = W ? 32 : kNS * 32;
        const int lo0 = (r_range & 0xffff) - wave * kWaveKeys;
        const int hi0 = EXTRA ? (r_range >> 16) - wave * kWaveKeys : kWaveKeys;
        if (do_stats) {
            const uint32_t wstats_ad = lds0 + kOffWstats + PAR * kWstatsBytes + wave * (kMaxRowsF * 8) + ((uint32_t)(lane & 31) << 3);
            stats_pass<NB * GB, PAR, W, F8>(c_stats, ring.kf[SLOT], lc, sub_slot_off(wave, wk.slot0, 0),
                                     sub_slot_off(wave, wk.slot0, 1), wstats_ad, lo0, hi0, lane, ki, voff, lse_row,
                                     look_row, a.rows_pad, lds0 + kOffXlse);
        } else {
            if (lse_row != nullptr) stage_exchange_rows(lds0 + kOffXlse, lse_row, look_row, a.rows_pad, lane);
            k_issue<kSI>(ki, voff, 0);
        }
    }

    // ---- pre-barrier: exchange data in, seeds out ----
    if (wave == kLseWave) vm_wait<kLoadsBehindLse<NB * GB, F8>>(); else vm_wait<2 * kSI>();
    int *fail = reinterpret_cast<int *>(lds + kOffFail);
    if (wave == kDutyWave) {
        if (duty_blk >= 0) {
            uint32_t row_mask = 0;
#pragma unroll
            for (int r = 0; r < kDutyRows; ++r) {
                int g, n;
                if (row_valid<NB>(a, duty_blk * kDutyRows + r, g, n)) row_mask |= 1u << r;
            }
            if (row_mask != 0) {
                const uint32_t par = (uint32_t)(pd / kSlots) & 1u;
                const uint64_t *src = a.part + ((size_t)(pd % kSlots) * a.n_wg + src_w0) * a.rows_pad + duty_blk * kDutyRows;
                // fast path: the partials requested at the start of this step are all there; otherwise poll (bounded)
                DutyBlock de = read_duty_staging(lds0, lane);
                bool ready = !__any(!duty_ready(de, par, lane, src_n, row_mask)) && a.force_miss == 0;
                if (!ready && *fail == 0) {
                    unsigned spins = 0;
                    do {
                        if (++spins > a.spin_max) { raise_failure(a, fail); break; }
#pragma unroll
                        for (int r = 0; r < kDutyRows; ++r)
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                de.e[r][q] = ld64(src + (size_t)min(lane + 64 * q, src_n - 1) * a.rows_pad + r);
                        ready = !__any(!duty_ready(de, par, lane, src_n, row_mask)) && a.force_miss == 0;
                    } while (!ready);
                }
                // per row: maximum first, then one exponential per partial (short dependency chains, fixed order)
                float mine = 0.f;       // lane r keeps the normaliser of row r of the block
#pragma unroll
                for (int r = 0; r < kDutyRows; ++r) {
                    float pm[4], pl4[4], m = neg_inf();
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const bool valid = lane + 64 * q < src_n;
                        pm[q] = valid ? __uint_as_float((uint32_t)de.e[r][q]) : neg_inf();
                        pl4[q] = valid ? __uint_as_float((uint32_t)(de.e[r][q] >> 32) & 0x7fffffffu) : 0.f;
                        m = fmaxf(m, pm[q]);
                    }
                    m = wave_max(m);
                    float l = 0.f;
#pragma unroll
                    for (int q = 0; q < 4; ++q) l += pl4[q] * fast_exp2((pm[q] - m) * c_duty);
                    l = wave_sum(l);
                    const float v = -(m + fast_log2(l) * (F8 ? 1.0f / c_duty : a.inv_c));
                    if (lane == r) mine = v;
                }
                // a duty that could not be completed (now or because the workgroup has failed before)
                // publishes poison: whoever reads it fails too instead of using a wrong normaliser
                const uint32_t tag = (ready && *fail == 0) ? (uint32_t)(pd + 1) : kPoisonTag;
                if (lane < kDutyRows && ((row_mask >> lane) & 1u))
                    st64(a.lse + ((size_t)(pd % kSlots) * a.n_gp + lse_idx) * a.rows_pad + duty_blk * kDutyRows + lane,
                         (uint64_t)__float_as_uint(mine) | ((uint64_t)tag << 32));
            }
        }
    } else if (wave == kLseWave) {
        if (pl >= 0 && pl < n_phases && lane < a.rows_pad) {
            int g, n;
            float v = neg_inf();
            if (row_valid<NB>(a, lane, g, n)) {
                const uint64_t *src = a.lse + ((size_t)(pl % kSlots) * a.n_gp + a.p_idx) * a.rows_pad + lane;
                uint64_t entry = read_lse_staging(lds0, lane);
                if ((uint32_t)(entry >> 32) != (uint32_t)(pl + 1) && *fail == 0) {
                    unsigned spins = 0;
                    while ((uint32_t)(entry >> 32) != (uint32_t)(pl + 1)) {
                        if ((uint32_t)(entry >> 32) == kPoisonTag || ++spins > a.spin_max) { raise_failure(a, fail); break; }
                        entry = ld64(src);
                    }
                }
                v = __uint_as_float((uint32_t)entry);
                if (EXTRA && a.look != nullptr) {
                    // the row's softmax also runs over its visible lookahead keys: log-sum-exp of the
                    // prompt's normaliser and theirs (-inf when the row sees none), in raw-logit units
                    const float lp = -v, lk = read_look_staging(lds0, lane), top = fmaxf(lp, lk);
                    v = -(top + fast_log2(fast_exp2((lp - top) * a.c) + fast_exp2((lk - top) * a.c)) * a.inv_c);
                }
            }
            const int rho = lane & 31;
            lds_store_f32(lds0 + kOffCinit + PAR * (kMaxRowsF * 4) +
                              4u * (uint32_t)((lane & ~31) + ((rho >> 2) & 1) * 16 + 4 * (rho >> 3) + (rho & 3)), v);
        }
    }

    // ---- walk on ----
    if (s + 2 < n_phases) {               // K pointer of the next step's fetch
        if (++wk.k.kv == a.n_kv_heads) {
            wk.k.kv = 0;
            ++wk.k.layer;
            wk.kptr = reinterpret_cast<const char *>(kp.p[wk.k.layer]) + wave_off;
        } else {
            wk.kptr += (uint64_t)a.k_stride_head * kElem;
        }
    }
    phase_advance(wk.c, s - 3, n_phases, a.n_kv_heads);
    wk.slot0 = slot_next;
    if (s - 1 > 0 && s - 1 < n_phases) {
        wk.dfirst += (a.rows_pad / kDutyRows) * a.n_gp;
        if (wk.dfirst >= a.n_wg) wk.dfirst -= a.n_wg;
    }
    lds_barrier();
}

// Model shapes. The kernel takes every dimension at run time (AnyModel); an instantiation for a
// fixed model overwrites its copy of the arguments with the model's constants, which the compiler
// then folds: fewer live scalars (the generic kernel spills some sixty of them) and no address
// arithmetic on run-time dimensions. Prompt length, workgroup count, kv-head stride and pointers
// stay run-time values; the workgroup count is folded too in the instantiations for a prompt that
// fills the device (256 workgroups: 128K tokens), where every exchange slot is in use and the bounds
// checks on workgroup indices fall away.
struct AnyModel {
    static constexpr bool kFixed = false;
    static constexpr int kLayers = 0, kQHeads = 0, kKvHeads = 0, kNq = 0, kWorkgroups = 0;
};
// The 16-layer, 32-query / 8-kv-head, head_dim 64 draft shape (a Llama-3.2-1B-class draft; Table 1 of
// the paper) with NQ lookahead rows, token-contiguous keys and scale 1/8.
template <int NQ, int WORKGROUPS>
struct Draft16x32x8 {
    static constexpr bool kFixed = true;
    static constexpr int kLayers = 16, kQHeads = 32, kKvHeads = 8, kNq = NQ, kWorkgroups = WORKGROUPS;   // 0: run-time count
};
constexpr float kScaleEighthLog2e = 0.125f * 1.44269504088896340736f;    // scale 1/sqrt(64) times log2(e), as the host computes it

template <class M>
__device__ __forceinline__ void fold_model_constants(FusedArgs &a)
{
    if (M::kFixed) {
        a.n_layers = M::kLayers;
        a.n_q_heads = M::kQHeads;
        a.n_kv_heads = M::kKvHeads;
        a.group = M::kQHeads / M::kKvHeads;
        a.n_q = M::kNq;
        a.n_nblk = (M::kNq + 7) / 8;
        a.n_gblk = (M::kQHeads / M::kKvHeads + 3) / 4;
        a.rows_pad = a.n_nblk * a.n_gblk * 32;
        a.k_stride_token = kD;
        a.c = kScaleEighthLog2e;
        a.inv_c = 1.0f / kScaleEighthLog2e;
        if (M::kWorkgroups > 0) a.n_wg = M::kWorkgroups;
    }
}

// W: head_dim 128. A workgroup owns 256 keys, a wave 32; the two "sub-tiles" of a wave are the two
// 64-element halves of its keys' rows (same transit ring, same fragment ring: kf[s][t] holds MFMA
// k-step 4s + t), Q tiles hold 32 rows as two half-tiles, and a logit is one chain of eight MFMA steps.
// F8: 8-bit keys (head_dim 64): rows of 64 codes, sub-tiles of 2 KB fetched by two instructions of 16 rows,
// widened to bf16 at the lift; every phase has its own key scale.
template <int NB, int GB, bool EXTRA, class M, bool W = false, bool F8 = false>
__global__ __launch_bounds__(kFThreads, 2) void sp_fused_kernel(FusedArgs a, LayerPtrs kp, GroupTable gt)
{
    static_assert(!W || (NB == 1 && GB == 1 && !M::kFixed), "head_dim 128: one block of 32 query rows");
    static_assert(!F8 || !EXTRA, "8-bit keys: plain variants only");
    constexpr int kSI = F8 ? kSubInstr / 2 : kSubInstr;
    constexpr uint32_t kElem = F8 ? 1u : 2u;
    constexpr int kTile = W ? kFTile / 2 : kFTile;            // keys per workgroup
    constexpr int kWaveKeys = kTile / kFWaves;
    constexpr int kHeadDim = W ? 2 * kD : kD;
    __shared__ __attribute__((aligned(1024))) unsigned char lds[kLdsBytes];
    fold_model_constants<M>(a);

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, hf = lane >> 5, col = lane & 31;
    const int w = blockIdx.x;
    const int n_phases = a.n_layers * a.n_kv_heads;
    // Contiguous keys: the last workgroup's tile is shifted back so that it ends with the prompt (the
    // caller guarantees L >= 512): every workgroup loads 512 real keys; rows below r_lo belong to the
    // previous workgroup. Paged keys: pages are allocated whole and hold a multiple of 512 keys, so the
    // last tile stays where it is and rows from r_hi on (allocated, never written) are ignored.
    // Several prompts in one launch (their keys packed back to back, every prompt at least one tile long):
    // prompt p owns workgroups gt.w0[p] .. gt.w0[p+1]-1 and is a prompt of its own in everything
    // below: tile positions count from its first key, its queries are its own, partials are combined
    // among its workgroups only and its normalisers have their own row.
    const bool paged = EXTRA && a.block_table != nullptr;
    int64_t p_start = 0, p_len = a.L;
    int wl = w;                               // this workgroup's index within its prompt
    if (EXTRA && gt.n > 0) {
        int p = 0;
        while (p + 1 < gt.n && w >= gt.w0[p + 1]) ++p;
        p_start = gt.start[p];
        p_len = gt.len[p];
        wl = w - gt.w0[p];
        a.q += (size_t)gt.prompt[p] * ((size_t)a.n_layers * a.n_q_heads * a.n_q * kHeadDim);
        a.p_idx = p;
        a.n_gp = gt.n;
    } else {
        a.p_idx = 0;
        a.n_gp = 1;
    }
    const int64_t j0l = (paged || (int64_t)(wl + 1) * kTile <= p_len) ? (int64_t)wl * kTile : p_len - kTile;
    const int64_t j0 = p_start + j0l;         // first key of the tile in the layer's key array
    const int r_lo = (int)((int64_t)wl * kTile - j0l);
    const int r_hi = (int)(p_len - j0l < kTile ? p_len - j0l : kTile);
    const int r_range = r_lo | (r_hi << 16);
    const uint32_t lds0 = lds_addr(lds);
    const uint32_t stride_bytes = (uint32_t)a.k_stride_token * kElem;

    // zero the Q tiles (their padding rows are never loaded), seed the accumulator seeds with -inf
    {
        u32x4 *z = reinterpret_cast<u32x4 *>(lds + kOffQ1);
        const u32x4 zero = {0u, 0u, 0u, 0u};
        for (int i = tid; i < 4 * kQTileBytes / 16; i += kFThreads) z[i] = zero;
        float *ci = reinterpret_cast<float *>(lds + kOffCinit);
        if (tid < 2 * kMaxRowsF) ci[tid] = neg_inf();
        if (tid == 0) *reinterpret_cast<int *>(lds + kOffFail) = 0;
    }
    __syncthreads();

    LaneConst lc;
#pragma unroll
    for (int t = 0; t < kKS; ++t) lc.ld[t] = lds0 + 16u * (uint32_t)lds_slot<kD>(col, 2 * t + hf);
    // 8-bit sub-tile: row r at 64 r, its four 16-byte chunks XOR-swizzled by (r >> 2) & 3 (eight-byte reads of
    // 64 lanes then spread over all banks twice, which is what 512 bytes need anyway)
#pragma unroll
    for (int t = 0; t < kKS; ++t) lc.ld8[t] = lds0 + 64u * (uint32_t)col + ((((uint32_t)t ^ ((uint32_t)col >> 2)) & 3u) << 4) + 8u * (uint32_t)hf;
    {
        uint32_t rowpart = (uint32_t)(lane >> 3) * stride_bytes;
        const uint32_t swz = (uint32_t)(lane >> 4);               // (row >> 1) & 7 of row = lane >> 3 in an even instruction
        lc.koff[0] = rowpart + (((uint32_t)(lane & 7) ^ swz) << 4);
        lc.koff[1] = rowpart + (((uint32_t)(lane & 7) ^ (swz | 4u)) << 4);
        if (F8) {       // an instruction moves 16 rows of 64 bytes: row lane >> 2, chunk (lane & 3) ^ ((row >> 2) & 3)
            rowpart = (uint32_t)(lane >> 2) * stride_bytes;
            lc.koff[0] = lc.koff[1] = rowpart + ((((uint32_t)lane & 3u) ^ (((uint32_t)lane >> 4) & 3u)) << 4);
        }
        // a wave's slice of a Q tile: 8 rows (W: of one half-tile, waves 4..7 take the second halves)
        const int row = (W ? (wave & 3) : wave) * 8 + (lane >> 3);
        int g, n;
        lc.qoff = -1;
        if (row < a.rows_pad && row_valid<NB>(a, row, g, n))
            lc.qoff = ((g * a.n_q + n) * kHeadDim + (W ? (wave >> 2) * kD : 0) + (((lane & 7) ^ ((row >> 1) & 7)) << 3)) * 2;
    }

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

    // byte offset of this wave's first key within a (layer, kv head): uniform, kept in scalar registers
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    uint64_t wave_off = (uint64_t)(j0 + wave_u * kWaveKeys) * (uint64_t)a.k_stride_token * kElem;
    if (paged) {
        const int64_t page = j0 / a.page_tokens;
        wave_off = ((uint64_t)a.block_table[page] * (uint64_t)a.page_stride +
                    (uint64_t)(j0 - page * a.page_tokens + wave_u * kWaveKeys) * (uint64_t)a.k_stride_token) * 2u;
    }
    wave_off = (uint64_t)uniform32((uint32_t)wave_off) | ((uint64_t)uniform32((uint32_t)(wave_off >> 32)) << 32);

    // prologue: this wave's slice of Q(0) and both sub-tiles of K(0); everything lands before step 0
    if (lc.qoff >= 0) dma_u<kOffQ1>((uint32_t)lc.qoff, a.q, lds0 + wave_u * 1024);
#pragma unroll
    for (int s2 = 0; s2 < kNS; ++s2) {
        KIssue ki;
        ki.lds_dst = lds0 + sub_slot_off(wave_u, 0, s2);
        ki.base = reinterpret_cast<const char *>(kp.p[0]) + wave_off + (W ? (uint64_t)(s2 * kD * kElem) : (uint64_t)(s2 * 32) * stride_bytes);
        ki.step_bytes = (F8 ? 16u : 8u) * stride_bytes;
        k_issue<kSI>(ki, lc.koff, 0);
    }
    vm_wait<0>();
    lds_barrier();

    Walk wk;
    wk.k = phase_at(1, n_phases, a.n_kv_heads);
    wk.kptr = reinterpret_cast<const char *>(kp.p[wk.k.layer]) + (uint64_t)wk.k.kv * (uint64_t)a.k_stride_head * kElem + wave_off;
    wk.c = phase_at(0, n_phases, a.n_kv_heads);
    wk.slot0 = 0;
    wk.dfirst = 0;
    if (!EXTRA) { a.p_idx = 0; a.n_gp = 1; }

    // The body is unrolled four times so that the fragment ring slot (s % 4) and the buffer parity
    // (s % 2) are compile-time; the trip count is rounded up, surplus steps do no work but keep the
    // instruction stream uniform. The last probability pass (phase n_phases - 1) runs in step n_phases + 3.
    const int n_steps = (n_phases + kLag + 1 + 3) / 4 * 4;
    for (int s0 = 0; s0 < n_steps; s0 += 4) {
        step<NB, GB, 0, 0, EXTRA, W, F8>(a, kp, gt, s0 + 0, n_phases, ring, acc, lc, wk, lds, lds0, wave_off, r_range);
        step<NB, GB, 1, 1, EXTRA, W, F8>(a, kp, gt, s0 + 1, n_phases, ring, acc, lc, wk, lds, lds0, wave_off, r_range);
        step<NB, GB, 2, 0, EXTRA, W, F8>(a, kp, gt, s0 + 2, n_phases, ring, acc, lc, wk, lds, lds0, wave_off, r_range);
        step<NB, GB, 3, 1, EXTRA, W, F8>(a, kp, gt, s0 + 3, n_phases, ring, acc, lc, wk, lds, lds0, wave_off, r_range);
    }
    vm_wait<0>();               // no direct-to-LDS load may outlive the workgroup
    lds_barrier();
    // the call has failed if any workgroup raised the status word; this workgroup's own failures are in it
    const bool failed = __hip_atomic_load(a.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u;
#pragma unroll
    for (int s = 0; s < kWaveKeys / 32; ++s) {
        const float both = acc.total[s] + __shfl_xor(acc.total[s], 32);
        const int key = wave * kWaveKeys + s * 32 + col;
        if (hf == 0 && key >= r_lo && key < r_hi) a.scores[j0 + key] = failed ? __uint_as_float(0x7fc00000u) : both * a.out_scale;   // quiet NaN marks a failed call
    }
}

// Clears the exchange area and the status word: a zero sum marks a partial as not yet written and
// phase numbers start at 1, so zero normaliser entries are never taken as ready.
__global__ void sp_fused_clear_kernel(uint64_t *p, size_t n, uint32_t *err)
{
    if (err != nullptr && blockIdx.x == 0 && threadIdx.x == 0) *err = 0u;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0;
}

// Test hook (see sp_debug_fused_giveup): polls before a wait gives up, and whether duty waves treat
// their partials as never arriving.
std::atomic<uint32_t> g_spin_max{1u << 20};     // about a second
std::atomic<int32_t> g_force_miss{0};

}  // namespace

namespace sp_fused {

void set_giveup(uint32_t spin_max, int32_t force_miss)
{
    g_spin_max.store(spin_max, std::memory_order_relaxed);
    g_force_miss.store(force_miss, std::memory_order_relaxed);
}

size_t workspace_bytes(int rows_pad, int n_wg, int n_prompts)
{
    return sp::align_up(sizeof(uint64_t) * ((size_t)kSlots * rows_pad * n_wg + (size_t)kSlots * rows_pad * n_prompts), 256);
}

bool fits_one_per_cu()
{
    int n1 = 0, n2 = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n1, sp_fused_kernel<1, 1, true, AnyModel>, kFThreads, 0) != hipSuccess) return false;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n2, sp_fused_kernel<2, 1, true, AnyModel>, kFThreads, 0) != hipSuccess) return false;
    return n1 >= 1 && n2 >= 1;
}

sp_status launch(FusedArgs a, const LayerPtrs &kp, const GroupTable *group, bool clear_status, void *ws,
                 uint32_t *status_word, hipStream_t st)
{
    GroupTable gt;
    std::memset(&gt, 0, sizeof gt);
    if (group) gt = *group;
    // The kernel places workgroup w of a prompt at key w * tile: the grid must be exactly the prompts' tiles
    // (a surplus workgroup of a paged prompt would look up a page the table does not have).
    const int64_t tile = a.tile_keys;
    if (!(a.head_dim == kD && tile == kFTile) && !(a.head_dim == 2 * kD && tile == kFTile / 2))
        return sp::fail(SP_ERR_INVALID_ARG, "fused score kernel: head_dim %d with %d keys per workgroup", a.head_dim, a.tile_keys);
    if (gt.n == 0) {
        if (a.L < tile || sp::ceil_div(a.L, tile) != a.n_wg)
            return sp::fail(SP_ERR_INVALID_ARG, "fused score kernel: %d workgroups for %lld keys", a.n_wg, (long long)a.L);
    } else {
        if (gt.n < 0 || gt.n > sp_fused::kMaxGroupPrompts || gt.w0[0] != 0 || gt.w0[gt.n] != a.n_wg)
            return sp::fail(SP_ERR_INVALID_ARG, "fused score kernel: group table does not cover %d workgroups", a.n_wg);
        for (int i = 0; i < gt.n; ++i)
            if (gt.len[i] < tile || sp::ceil_div(gt.len[i], tile) != gt.w0[i + 1] - gt.w0[i])
                return sp::fail(SP_ERR_INVALID_ARG, "fused score kernel: prompt %d of the group: %d workgroups for %lld keys", i,
                                gt.w0[i + 1] - gt.w0[i], (long long)gt.len[i]);
    }
    uint64_t *base = static_cast<uint64_t *>(ws);
    const size_t n_part = (size_t)kSlots * a.rows_pad * a.n_wg, n_lse = (size_t)kSlots * a.rows_pad * (gt.n > 0 ? gt.n : 1);
    a.part = base;
    a.lse = base + n_part;
    a.err = status_word;
    a.spin_max = g_spin_max.load(std::memory_order_relaxed);
    a.force_miss = g_force_miss.load(std::memory_order_relaxed);
    const size_t n_clear = n_part + n_lse;
    hipLaunchKernelGGL(sp_fused_clear_kernel, dim3((unsigned)((n_clear + 255) / 256 > 1024 ? 1024 : (n_clear + 255) / 256)),
                       dim3(256), 0, st, base, n_clear, clear_status ? status_word : (uint32_t *)nullptr);
    SP_HIP_CHECK(hipGetLastError());
    // Every workgroup must be resident for the exchange to make progress: one workgroup fits per
    // compute unit (LDS), so the grid may not exceed the number of compute units. All waits in the
    // kernel are bounded; should residency fail (the device shared with other work), the call ends
    // with NaN scores and the status word set instead of hanging.
    const bool extra = a.look != nullptr || a.block_table != nullptr || gt.n > 0;
    const dim3 grid(a.n_wg), block(kFThreads);
    if (a.kscale != nullptr) {              // 8-bit keys
        if (extra) return sp::fail(SP_ERR_UNSUPPORTED, "fused score kernel, 8-bit keys: one prompt, contiguous keys only");
        if (a.head_dim == 2 * kD) {
            if (a.n_nblk != 1 || a.n_gblk != 1)
                return sp::fail(SP_ERR_UNSUPPORTED, "fused score kernel, head_dim 128: %d x %d row blocks", a.n_nblk, a.n_gblk);
            hipLaunchKernelGGL((sp_fused_kernel<1, 1, false, AnyModel, true, true>), grid, block, 0, st, a, kp, gt);
            SP_HIP_CHECK(hipGetLastError());
            return SP_OK;
        }
        const bool draft8 = a.n_layers == 16 && a.n_q_heads == 32 && a.n_kv_heads == 8 && a.k_stride_token == kD &&
                            a.c == kScaleEighthLog2e && a.inv_c == 1.0f / kScaleEighthLog2e;
        if (draft8 && a.n_q == 16 && a.n_wg == 256) hipLaunchKernelGGL((sp_fused_kernel<2, 1, false, Draft16x32x8<16, 256>, false, true>), grid, block, 0, st, a, kp, gt);
        else if (draft8 && a.n_q == 16) hipLaunchKernelGGL((sp_fused_kernel<2, 1, false, Draft16x32x8<16, 0>, false, true>), grid, block, 0, st, a, kp, gt);
        else if (draft8 && a.n_q == 8) hipLaunchKernelGGL((sp_fused_kernel<1, 1, false, Draft16x32x8<8, 0>, false, true>), grid, block, 0, st, a, kp, gt);
        else if (a.n_nblk == 2 && a.n_gblk == 1) hipLaunchKernelGGL((sp_fused_kernel<2, 1, false, AnyModel, false, true>), grid, block, 0, st, a, kp, gt);
        else if (a.n_nblk == 1 && a.n_gblk == 2) hipLaunchKernelGGL((sp_fused_kernel<1, 2, false, AnyModel, false, true>), grid, block, 0, st, a, kp, gt);
        else if (a.n_nblk == 1 && a.n_gblk == 1) hipLaunchKernelGGL((sp_fused_kernel<1, 1, false, AnyModel, false, true>), grid, block, 0, st, a, kp, gt);
        else return sp::fail(SP_ERR_UNSUPPORTED, "fused score kernel: %d x %d row blocks", a.n_nblk, a.n_gblk);
        SP_HIP_CHECK(hipGetLastError());
        return SP_OK;
    }
    if (a.head_dim == 2 * kD) {
        if (a.n_nblk != 1 || a.n_gblk != 1)
            return sp::fail(SP_ERR_UNSUPPORTED, "fused score kernel, head_dim 128: %d x %d row blocks", a.n_nblk, a.n_gblk);
        if (extra) hipLaunchKernelGGL((sp_fused_kernel<1, 1, true, AnyModel, true>), grid, block, 0, st, a, kp, gt);
        else hipLaunchKernelGGL((sp_fused_kernel<1, 1, false, AnyModel, true>), grid, block, 0, st, a, kp, gt);
        SP_HIP_CHECK(hipGetLastError());
        return SP_OK;
    }
    // the fixed-model instantiations apply when every folded constant equals the call's value
    const bool draft_shape = a.kscale == nullptr && a.head_dim == kD && a.n_layers == 16 && a.n_q_heads == 32 && a.n_kv_heads == 8 && a.k_stride_token == kD &&
                             a.c == kScaleEighthLog2e && a.inv_c == 1.0f / kScaleEighthLog2e;
    const bool draft = !extra && draft_shape;
    const bool draft_batch = draft_shape && gt.n > 0 && a.look == nullptr && a.block_table == nullptr;    // several prompts a launch
    if (draft_batch && a.n_q == 16) {
        hipLaunchKernelGGL((sp_fused_kernel<2, 1, true, Draft16x32x8<16, 0>>), grid, block, 0, st, a, kp, gt);
    } else if (draft_batch && a.n_q == 8) {
        hipLaunchKernelGGL((sp_fused_kernel<1, 1, true, Draft16x32x8<8, 0>>), grid, block, 0, st, a, kp, gt);
    } else if (draft && a.n_q == 16) {
        if (a.n_wg == 256) hipLaunchKernelGGL((sp_fused_kernel<2, 1, false, Draft16x32x8<16, 256>>), grid, block, 0, st, a, kp, gt);
        else hipLaunchKernelGGL((sp_fused_kernel<2, 1, false, Draft16x32x8<16, 0>>), grid, block, 0, st, a, kp, gt);
    } else if (draft && a.n_q == 8) {
        if (a.n_wg == 256) hipLaunchKernelGGL((sp_fused_kernel<1, 1, false, Draft16x32x8<8, 256>>), grid, block, 0, st, a, kp, gt);
        else hipLaunchKernelGGL((sp_fused_kernel<1, 1, false, Draft16x32x8<8, 0>>), grid, block, 0, st, a, kp, gt);
    } else if (a.n_nblk == 2 && a.n_gblk == 1) {
        if (extra) hipLaunchKernelGGL((sp_fused_kernel<2, 1, true, AnyModel>), grid, block, 0, st, a, kp, gt);
        else hipLaunchKernelGGL((sp_fused_kernel<2, 1, false, AnyModel>), grid, block, 0, st, a, kp, gt);
    } else if (a.n_nblk == 1 && a.n_gblk == 2) {
        if (extra) hipLaunchKernelGGL((sp_fused_kernel<1, 2, true, AnyModel>), grid, block, 0, st, a, kp, gt);
        else hipLaunchKernelGGL((sp_fused_kernel<1, 2, false, AnyModel>), grid, block, 0, st, a, kp, gt);
    } else if (a.n_nblk == 1 && a.n_gblk == 1) {
        if (extra) hipLaunchKernelGGL((sp_fused_kernel<1, 1, true, AnyModel>), grid, block, 0, st, a, kp, gt);
        else hipLaunchKernelGGL((sp_fused_kernel<1, 1, false, AnyModel>), grid, block, 0, st, a, kp, gt);
    } else {
        return sp::fail(SP_ERR_UNSUPPORTED, "fused score kernel: %d x %d row blocks", a.n_nblk, a.n_gblk);
    }
    SP_HIP_CHECK(hipGetLastError());
    return SP_OK;
}

}  // namespace sp_fused

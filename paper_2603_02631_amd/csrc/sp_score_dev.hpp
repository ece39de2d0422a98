// Device-side pieces shared by the score kernels: vector types, the LDS tile
// layout, MFMA fragment loads and the log-sum-exp merge of row statistics.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace sp_dev {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kMaxLayers = 128;

struct LayerPtrs { const uint16_t *p[kMaxLayers]; };

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }
__device__ __forceinline__ float neg_inf() { return -__builtin_huge_valf(); }

// LDS tiles hold rows of D bf16 as D/8 chunks of 16 bytes; the chunk index is
// XOR-swizzled by the row so that 16 lanes reading one chunk column of 16
// consecutive rows hit 16 different bank groups.
template <int D>
__device__ __forceinline__ int lds_slot(int row, int chunk)
{
    constexpr int CH = D / 8;
    const int s = (CH == 8) ? ((row >> 1) & 7) : (row & 15);
    return row * CH + (chunk ^ s);
}

template <int D>
__device__ __forceinline__ void load_frag(const u32x4 *tile, int row, int hf, bf16x8 (&f)[D / 16])
{
#pragma unroll
    for (int t = 0; t < D / 16; ++t) f[t] = __builtin_bit_cast(bf16x8, tile[lds_slot<D>(row, 2 * t + hf)]);
}

// Eight E4M3 codes (two dwords) -> eight bf16 (every E4M3 value is exact in bf16: the upper half of
// its float image). Two conversions to fp32 pairs and two byte permutes per dword; the packed
// fp8 -> bf16 conversion of gfx950 gives the same bits in half the instructions but measured slower
// (0.569 against 0.529 ms for the single-launch kernel on 128K tokens).
__device__ __forceinline__ u32x4 e4m3x8_to_bf16x8(uint32_t c0, uint32_t c1)
{
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    u32x4 r;
    const uint32_t w[2] = {c0, c1};
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], false);     // codes 0, 1 of the dword
        const f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], true);      // codes 2, 3
        r[2 * i] = __builtin_amdgcn_perm(__float_as_uint(lo.y), __float_as_uint(lo.x), 0x07060302u);
        r[2 * i + 1] = __builtin_amdgcn_perm(__float_as_uint(hi.y), __float_as_uint(hi.x), 0x07060302u);
    }
    return r;
}

// (m, l) <- (m, l) (+) (m2, l2) for running softmax statistics in raw-logit units.
__device__ __forceinline__ void lse_merge(float &m, float &l, float m2, float l2, float c)
{
    const float mm = fmaxf(m, m2);
    if (mm == neg_inf()) { l = 0.f; return; }
    l = l * fast_exp2((m - mm) * c) + l2 * fast_exp2((m2 - mm) * c);
    m = mm;
}

}  // namespace sp_dev

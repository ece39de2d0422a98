// sp_hbm_read_probe: a plain streaming read of a device buffer, the measured ceiling next to the
// datasheet bandwidth that the score pass (one pass over the K cache; paper: Appendix A.1.1) is
// held against. No arithmetic beyond the XOR that keeps the loads alive.
#include "sp_common.hpp"

namespace {

constexpr int kProbeThreads = 256;
constexpr int kProbeUnroll = 8;              // 16-byte loads in flight per lane

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__global__ __launch_bounds__(kProbeThreads) void sp_probe_kernel(const u32x4 *__restrict__ p, size_t n16,
                                                                 unsigned long long *__restrict__ sink)
{
    // a block walks contiguous spans of kProbeThreads * kProbeUnroll chunks; consecutive lanes read
    // consecutive 16-byte chunks
    const size_t span = (size_t)kProbeThreads * kProbeUnroll;
    u32x4 acc = {0u, 0u, 0u, 0u};
    const size_t n_full = n16 / span * span;
    // whole spans: unconditional loads, all of a lane's loads in flight before the first is used
    for (size_t base = (size_t)blockIdx.x * span; base < n_full; base += (size_t)gridDim.x * span) {
        u32x4 v[kProbeUnroll];
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) v[u] = __builtin_nontemporal_load(p + base + (size_t)u * kProbeThreads + threadIdx.x);
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) acc ^= v[u];
    }
    // the ragged end of the buffer: one block, chunk by chunk
    if (blockIdx.x == 0)
        for (size_t i = n_full + threadIdx.x; i < n16; i += kProbeThreads) acc ^= p[i];
    unsigned long long x = ((unsigned long long)(acc.x ^ acc.z) << 32) | (unsigned long long)(acc.y ^ acc.w);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x ^= __shfl_xor(x, off);
    if ((threadIdx.x & 63) == 0) atomicXor(sink, x);
}

}  // namespace

extern "C" sp_status sp_hbm_read_probe(const void *buf_dev, size_t bytes, uint64_t *sink_dev, void *hip_stream)
{
    if (!buf_dev || !sink_dev) return sp::fail(SP_ERR_INVALID_ARG, "buf_dev and sink_dev must not be null");
    if (bytes == 0 || bytes % 16 != 0 || (uintptr_t)buf_dev % 16 != 0)
        return sp::fail(SP_ERR_INVALID_ARG, "the buffer must be 16-byte aligned and a positive multiple of 16 bytes long");
    static thread_local int cached_dev = -1, cached_cus = 0;     // the attribute query is slow next to a launch
    int dev = 0;
    SP_HIP_CHECK(hipGetDevice(&dev));
    if (dev != cached_dev) {
        SP_HIP_CHECK(hipDeviceGetAttribute(&cached_cus, hipDeviceAttributeMultiprocessorCount, dev));
        cached_dev = dev;
    }
    const int cus = cached_cus;
    const size_t n16 = bytes / 16;
    const size_t span = (size_t)kProbeThreads * kProbeUnroll;
    size_t blocks = (n16 + span - 1) / span;
    const size_t cap = (size_t)(cus > 0 ? cus : 256) * 8;           // eight workgroups per compute unit
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(sp_probe_kernel, dim3((unsigned)blocks), dim3(kProbeThreads), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const u32x4 *>(buf_dev), n16, reinterpret_cast<unsigned long long *>(sink_dev));
    SP_HIP_CHECK(hipGetLastError());
    return SP_OK;
}

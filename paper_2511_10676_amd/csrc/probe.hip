// Device ceilings, measured rather than quoted: a streaming read and a
// register-only matrix-instruction loop.  They are measurement aids for the
// benchmark (what this device delivers for the two resources the predict
// kernels are bound by), not part of the method.
//
//   read   every workgroup streams a contiguous span with 16-byte loads per
//          lane, eight in flight (a perfectly coalesced stream), xors what it
//          read and writes one word per wave so the loads cannot be dropped.
//   mfma   every wave issues v_mfma_f32_32x32x16_bf16 on eight independent
//          accumulators from operands that stay in registers: no memory, no
//          LDS, two waves per SIMD on every CU.  What comes out is the matrix
//          peak at the clock the chip sustains under that load.
#include "paep_device.h"
#include "paep_internal.h"

namespace paep {

static constexpr int PROBE_THREADS = 256;

__global__ __launch_bounds__(PROBE_THREADS) void probe_read_kernel(const u32x4* __restrict__ src, long long n16,
                                                                   long long span16, uint32_t* __restrict__ sink)
{
    // workgroup b owns the contiguous span [b * span16, (b + 1) * span16) of 16-byte words
    const long long lo = (long long)blockIdx.x * span16;
    const long long hi = lo + span16 < n16 ? lo + span16 : n16;
    long long i = lo + threadIdx.x;
    u32x4 acc = u32x4{0u, 0u, 0u, 0u};
    for (; i + 7 * PROBE_THREADS < hi; i += 8 * PROBE_THREADS) {         // eight loads in flight per lane
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[i + u * PROBE_THREADS];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
    }
    for (; i < hi; i += PROBE_THREADS) acc ^= src[i];
    uint32_t v = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) v ^= __shfl_xor(v, m, 64);
    if ((threadIdx.x & 63) == 0) sink[blockIdx.x * (PROBE_THREADS / 64) + (threadIdx.x >> 6)] = v;
}

__global__ __launch_bounds__(512, 1) void probe_mfma_kernel(int iters, float* __restrict__ sink)
{
    const int lane = threadIdx.x & 63;
    // operands: small exact values so the accumulators stay finite
    u32x4 abits = u32x4{0x3C003C00u + (uint32_t)lane, 0x3C003C00u, 0x3C003C00u, 0x3C003C00u};
    const bf16x8 a = __builtin_bit_cast(bf16x8, abits);
    const bf16x8 b = __builtin_bit_cast(bf16x8, u32x4{0x3B803B80u, 0x3B803B80u, 0x3B803B80u, 0x3B803B80u});
    f32x16 acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) s += acc[j][0] + acc[j][15];
    if (s == 12345.678f) sink[blockIdx.x] = s;              // never true; keeps the loop alive
}

hipError_t launch_probe_read(const void* src, size_t bytes, void* sink, hipStream_t stream)
{
    // sink: 4 bytes per wave, PROBE_READ_GROUPS workgroups of four waves
    // spans of 256 KB (the amount one decode workgroup streams), longer when that would need too many workgroups
    const long long n16 = (long long)(bytes / 16);
    long long span16 = (256 << 10) / 16;
    if (n16 > span16 * PROBE_READ_GROUPS) span16 = (n16 + PROBE_READ_GROUPS - 1) / PROBE_READ_GROUPS;
    const long long groups = (n16 + span16 - 1) / span16;
    if (groups == 0) return hipSuccess;
    hipLaunchKernelGGL(probe_read_kernel, dim3((unsigned)groups), dim3(PROBE_THREADS), 0, stream,
                       (const u32x4*)src, n16, span16, (uint32_t*)sink);
    return hipGetLastError();
}

hipError_t launch_probe_mfma(int groups, int iters, void* sink, hipStream_t stream)
{
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(groups), dim3(512), 0, stream, iters, (float*)sink);
    return hipGetLastError();
}

}  // namespace paep

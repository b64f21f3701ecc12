// Accuracy counters of the paper's section 5.1: exact match, correctly
// predicted experts, over-provisioning hit, top-1.  One thread per token row
// builds two bitsets over the expert ids (prediction and label), so set
// semantics come for free; rows are reduced per wave with shuffles and added
// to the layer's four 64-bit counters with integer atomics (exact, hence
// deterministic).  A first tiny launch clears the counters.
#include "paep_internal.h"

namespace paep {

static constexpr int SCORE_THREADS = 256;

__global__ void score_clear_kernel(unsigned long long* counters, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) counters[i] = 0ull;
}

template <int NW>   // 64-bit words per bitset: E <= 64 * NW
__global__ __launch_bounds__(SCORE_THREADS) void score_kernel(
    const int32_t* __restrict__ idx, int k_pred, const int32_t* __restrict__ ref, int k_ref,
    int T, int E, unsigned long long* __restrict__ counters)
{
    const int layer = blockIdx.y;
    const int t = blockIdx.x * SCORE_THREADS + threadIdx.x;
    int exact = 0, hit = 0, cover = 0, top1 = 0;
    if (t < T) {
        const int32_t* p = idx + ((long long)layer * T + t) * k_pred;
        const int32_t* q = ref + ((long long)layer * T + t) * k_ref;
        uint64_t P[NW], R[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) { P[w] = 0; R[w] = 0; }
        bool ok = true;
        for (int j = 0; j < k_pred; ++j) {
            const int e = p[j];
            ok = ok && (e >= 0 && e < E);
            const uint64_t bit = 1ull << (e & 63);
#pragma unroll
            for (int w = 0; w < NW; ++w) P[w] |= ((e >> 6) == w) ? bit : 0ull;
        }
        for (int j = 0; j < k_ref; ++j) {
            const int e = q[j];
            ok = ok && (e >= 0 && e < E);
            const uint64_t bit = 1ull << (e & 63);
#pragma unroll
            for (int w = 0; w < NW; ++w) R[w] |= ((e >> 6) == w) ? bit : 0ull;
        }
        if (ok) {
            int nP = 0, nR = 0, both = 0;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                nP += __popcll(P[w]);
                nR += __popcll(R[w]);
                both += __popcll(P[w] & R[w]);
            }
            hit = both;
            cover = (both == nR);
            exact = (both == nR && both == nP);
            const int e0 = p[0];
            uint64_t word = 0;
#pragma unroll
            for (int w = 0; w < NW; ++w) word = ((e0 >> 6) == w) ? R[w] : word;
            top1 = (int)((word >> (e0 & 63)) & 1ull);
        }
    }
    // wave reduction, then one atomic per wave and counter
    int packed_small = exact | (cover << 8) | (top1 << 16);    // each <= 64 after the reduction
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
        packed_small += __shfl_xor(packed_small, m, 64);
        hit += __shfl_xor(hit, m, 64);
    }
    if ((threadIdx.x & 63) == 0) {
        unsigned long long* c = counters + (long long)layer * 4;
        const int ex = packed_small & 0xFF, cv = (packed_small >> 8) & 0xFF, t1 = (packed_small >> 16) & 0xFF;
        if (ex) atomicAdd(&c[0], (unsigned long long)ex);
        if (hit) atomicAdd(&c[1], (unsigned long long)hit);
        if (cv) atomicAdd(&c[2], (unsigned long long)cv);
        if (t1) atomicAdd(&c[3], (unsigned long long)t1);
    }
}

hipError_t launch_score(const int32_t* idx, int k_pred, const int32_t* ref, int k_ref,
                        int L, int T, int E, long long* counters, hipStream_t stream)
{
    unsigned long long* c = (unsigned long long*)counters;
    hipLaunchKernelGGL(score_clear_kernel, dim3((4 * L + 255) / 256), dim3(256), 0, stream, c, 4 * L);
    if (T > 0) {
        dim3 grid((T + SCORE_THREADS - 1) / SCORE_THREADS, L);
        if (E <= 64)
            hipLaunchKernelGGL(score_kernel<1>, grid, dim3(SCORE_THREADS), 0, stream, idx, k_pred, ref, k_ref, T, E, c);
        else if (E <= 256)
            hipLaunchKernelGGL(score_kernel<4>, grid, dim3(SCORE_THREADS), 0, stream, idx, k_pred, ref, k_ref, T, E, c);
        else
            hipLaunchKernelGGL(score_kernel<16>, grid, dim3(SCORE_THREADS), 0, stream, idx, k_pred, ref, k_ref, T, E, c);
    }
    return hipGetLastError();
}

}  // namespace paep

// Expert popularity of each layer from its activation counts: the experts
// ordered by how often they were selected (the order a popularity-driven
// prefetcher loads them in, paper section 2.2.2) and the normalised Shannon
// entropy of the activation distribution (section 2.1, where 0.976 is reported
// for near-uniform routing).
//
// One workgroup per layer; E <= 1024 values, so everything lives in LDS.
// Rank by counting: expert e goes to position #{e' : key(e') > key(e)} with
// key = (count, lower id first), which needs no sorting network and is the
// same for any schedule.  The entropy is summed in double in a fixed order
// (strided partial sums per thread, then a tree over the threads).
#include "paep_internal.h"

namespace paep {

static constexpr int PROFILE_THREADS = 256;
static constexpr int PROFILE_MAX_E = 1024;

__global__ __launch_bounds__(PROFILE_THREADS) void activation_profile_kernel(
    const int32_t* __restrict__ counts, int E, int32_t* __restrict__ order, int32_t* __restrict__ n_active,
    double* __restrict__ entropy)
{
    __shared__ unsigned long long key[PROFILE_MAX_E];
    __shared__ double part[PROFILE_THREADS];
    __shared__ long long tot[PROFILE_THREADS];
    __shared__ int act[PROFILE_THREADS];
    const int layer = blockIdx.x, tid = threadIdx.x;
    const int32_t* c = counts + (long long)layer * E;
    int32_t* ord = order + (long long)layer * E;

    long long my_total = 0;
    int my_active = 0;
    for (int e = tid; e < E; e += PROFILE_THREADS) {
        const int32_t v = c[e] > 0 ? c[e] : 0;              // negative counts cannot come from grouping; treated as 0
        key[e] = ((unsigned long long)(uint32_t)v << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)e);
        my_total += v;
        my_active += (v > 0);
    }
    tot[tid] = my_total;
    act[tid] = my_active;
    __syncthreads();
    for (int s = PROFILE_THREADS / 2; s > 0; s >>= 1) {
        if (tid < s) { tot[tid] += tot[tid + s]; act[tid] += act[tid + s]; }
        __syncthreads();
    }
    const long long total = tot[0];
    const int nact = act[0];

    // popularity order: the active experts fill slots [0, nact), -1 the rest
    for (int e = tid; e < E; e += PROFILE_THREADS) {
        if (e >= nact) ord[e] = -1;
        const unsigned long long mine = key[e];
        if ((mine >> 32) == 0) continue;
        int rank = 0;
        for (int o = 0; o < E; ++o) rank += (key[o] > mine);
        ord[rank] = e;
    }

    // entropy = -sum p ln p / ln E
    double h = 0.0;
    if (E > 1 && total > 0) {
        for (int e = tid; e < E; e += PROFILE_THREADS) {
            const uint32_t v = (uint32_t)(key[e] >> 32);
            if (v > 0) {
                const double p = (double)v / (double)total;
                h -= p * log(p);
            }
        }
    }
    part[tid] = h;
    __syncthreads();
    for (int s = PROFILE_THREADS / 2; s > 0; s >>= 1) {
        if (tid < s) part[tid] += part[tid + s];
        __syncthreads();
    }
    if (tid == 0) {
        n_active[layer] = nact;
        entropy[layer] = (E > 1 && total > 0) ? part[0] / log((double)E) : 0.0;
    }
}

hipError_t launch_activation_profile(const int32_t* counts, int L, int E, int32_t* order, int32_t* n_active,
                                     double* entropy, hipStream_t stream)
{
    hipLaunchKernelGGL(activation_profile_kernel, dim3(L), dim3(PROFILE_THREADS), 0, stream, counts, E, order,
                       n_active, entropy);
    return hipGetLastError();
}

}  // namespace paep

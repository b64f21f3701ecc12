// Accuracy counters of the paper's section 5.1: exact match, correctly
// predicted experts, over-provisioning hit, top-1.  One thread per token row
// builds two bitsets over the expert ids (prediction and label), so set
// semantics come for free; rows are reduced per wave with shuffles and added
// to the layer's four 64-bit counters with integer atomics (exact, hence
// deterministic).  A first tiny launch clears the counters.  Short layers take
// a single launch instead: one workgroup per layer, no atomics.
#include "paep_internal.h"

namespace paep {

static constexpr int SCORE_THREADS = 256;

__global__ void score_clear_kernel(unsigned long long* counters, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) counters[i] = 0ull;
}

// One token row: bitsets of the predicted and the labelled experts.  The row's
// ids are fetched with independent loads (fixed trip count KM >= k) before any
// is looked at, so a row costs one memory round trip.
// Number of predicted ids row `row` uses: all k_pred, or its entry of k_row clamped to [1, k_pred].
__device__ __forceinline__ int row_width(const int32_t* __restrict__ k_row, long long row, int k_pred)
{
    if (!k_row) return k_pred;
    const int w = k_row[row];
    return w < 1 ? 1 : (w > k_pred ? k_pred : w);
}

template <int KM>
__device__ __forceinline__ void load_row(const int32_t* __restrict__ p, int k, int32_t (&v)[KM])
{
#pragma unroll
    for (int j = 0; j < KM; ++j) v[j] = (j < k) ? p[j] : 0;
}

template <int NW, int KM>   // 64-bit words per bitset: E <= 64 * NW; ids per row <= KM
__device__ __forceinline__ void score_vals(const int32_t (&pv)[KM], int k_pred, const int32_t (&qv)[KM], int k_ref,
                                           int E, int& exact, int& hit, int& cover, int& top1)
{
    uint64_t P[NW], R[NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) { P[w] = 0; R[w] = 0; }
    bool ok = true;
#pragma unroll
    for (int j = 0; j < KM; ++j) {
        if (j < k_pred) {
            const int e = pv[j];
            ok = ok && (e >= 0 && e < E);
            const uint64_t bit = 1ull << (e & 63);
#pragma unroll
            for (int w = 0; w < NW; ++w) P[w] |= ((e >> 6) == w) ? bit : 0ull;
        }
    }
#pragma unroll
    for (int j = 0; j < KM; ++j) {
        if (j < k_ref) {
            const int e = qv[j];
            ok = ok && (e >= 0 && e < E);
            const uint64_t bit = 1ull << (e & 63);
#pragma unroll
            for (int w = 0; w < NW; ++w) R[w] |= ((e >> 6) == w) ? bit : 0ull;
        }
    }
    if (!ok) return;                                        // a row with an id outside [0, E) scores nothing
    int nP = 0, nR = 0, both = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        nP += __popcll(P[w]);
        nR += __popcll(R[w]);
        both += __popcll(P[w] & R[w]);
    }
    hit += both;
    cover += (both == nR);
    exact += (both == nR && both == nP);
    const int e0 = pv[0];
    uint64_t word = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) word = ((e0 >> 6) == w) ? R[w] : word;
    top1 += (int)((word >> (e0 & 63)) & 1ull);
}

template <int NW, int KM>
__global__ __launch_bounds__(SCORE_THREADS) void score_kernel(
    const int32_t* __restrict__ idx, int k_pred, const int32_t* __restrict__ ref, int k_ref,
    int T, int E, const int32_t* __restrict__ k_row, unsigned long long* __restrict__ counters)
{
    const int layer = blockIdx.y;
    const int t = blockIdx.x * SCORE_THREADS + threadIdx.x;
    int exact = 0, hit = 0, cover = 0, top1 = 0;
    if (t < T) {
        int32_t pv[KM], qv[KM];
        const int kp = row_width(k_row, (long long)layer * T + t, k_pred);
        load_row<KM>(idx + ((long long)layer * T + t) * k_pred, kp, pv);
        load_row<KM>(ref + ((long long)layer * T + t) * k_ref, k_ref, qv);
        score_vals<NW, KM>(pv, kp, qv, k_ref, E, exact, hit, cover, top1);
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

// Up to LAYER_MAX_T tokens per layer: one workgroup per layer walks all rows,
// adds up inside the workgroup and stores the four counters -- one launch, no
// clearing pass and no atomics.
static constexpr int LAYER_THREADS = 1024;
static constexpr int LAYER_MAX_T = 1 << 12;

template <int NW, int KM>
__global__ __launch_bounds__(LAYER_THREADS) void score_layer_kernel(
    const int32_t* __restrict__ idx, int k_pred, const int32_t* __restrict__ ref, int k_ref,
    int T, int E, const int32_t* __restrict__ k_row, unsigned long long* __restrict__ counters)
{
    __shared__ int part[LAYER_THREADS / 64][4];
    const int layer = blockIdx.x, tid = threadIdx.x;
    int v[4] = {0, 0, 0, 0};                                // exact, hits, cover, top1; each < 2^31 (T*k bounded by the caller)
    // RU rows per thread at a time, all their loads issued before the first is used
    constexpr int RU = (KM <= 8) ? 4 : 1;
    for (int t0 = tid; t0 < T; t0 += LAYER_THREADS * RU) {
        int32_t pv[RU][KM], qv[RU][KM];
        int kp[RU];
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            const int t = t0 + u * LAYER_THREADS;
            kp[u] = k_pred;
            if (t < T) {
                kp[u] = row_width(k_row, (long long)layer * T + t, k_pred);
                load_row<KM>(idx + ((long long)layer * T + t) * k_pred, kp[u], pv[u]);
                load_row<KM>(ref + ((long long)layer * T + t) * k_ref, k_ref, qv[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < RU; ++u)
            if (t0 + u * LAYER_THREADS < T) score_vals<NW, KM>(pv[u], kp[u], qv[u], k_ref, E, v[0], v[1], v[2], v[3]);
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1)
#pragma unroll
        for (int c = 0; c < 4; ++c) v[c] += __shfl_xor(v[c], m, 64);
    if ((tid & 63) == 0)
#pragma unroll
        for (int c = 0; c < 4; ++c) part[tid >> 6][c] = v[c];
    __syncthreads();
    if (tid < 4) {
        unsigned long long sum = 0;
        for (int w = 0; w < LAYER_THREADS / 64; ++w) sum += (unsigned long long)part[w][tid];
        counters[(long long)layer * 4 + tid] = sum;
    }
}

template <int NW, int KM>
static void launch_score_cfg(const int32_t* idx, int k_pred, const int32_t* ref, int k_ref, int L, int T, int E,
                             const int32_t* k_row, unsigned long long* c, hipStream_t stream)
{
    if (T <= LAYER_MAX_T) {
        hipLaunchKernelGGL((score_layer_kernel<NW, KM>), dim3(L), dim3(LAYER_THREADS), 0, stream, idx, k_pred, ref,
                           k_ref, T, E, k_row, c);
        return;
    }
    hipLaunchKernelGGL(score_clear_kernel, dim3((4 * L + 255) / 256), dim3(256), 0, stream, c, 4 * L);
    dim3 grid((T + SCORE_THREADS - 1) / SCORE_THREADS, L);
    hipLaunchKernelGGL((score_kernel<NW, KM>), grid, dim3(SCORE_THREADS), 0, stream, idx, k_pred, ref, k_ref, T, E,
                       k_row, c);
}

hipError_t launch_score(const int32_t* idx, int k_pred, const int32_t* ref, int k_ref,
                        int L, int T, int E, const int32_t* k_row, long long* counters, hipStream_t stream)
{
    unsigned long long* c = (unsigned long long*)counters;
    const bool small_k = k_pred <= 8 && k_ref <= 8;         // the interface allows up to 32 ids per row
    if (E <= 64) {
        if (small_k) launch_score_cfg<1, 8>(idx, k_pred, ref, k_ref, L, T, E, k_row, c, stream);
        else         launch_score_cfg<1, 32>(idx, k_pred, ref, k_ref, L, T, E, k_row, c, stream);
    } else if (E <= 256) {
        if (small_k) launch_score_cfg<4, 8>(idx, k_pred, ref, k_ref, L, T, E, k_row, c, stream);
        else         launch_score_cfg<4, 32>(idx, k_pred, ref, k_ref, L, T, E, k_row, c, stream);
    } else {
        if (small_k) launch_score_cfg<16, 8>(idx, k_pred, ref, k_ref, L, T, E, k_row, c, stream);
        else         launch_score_cfg<16, 32>(idx, k_pred, ref, k_ref, L, T, E, k_row, c, stream);
    }
    return hipGetLastError();
}

// Confidence-driven over-provisioning (the paper's closing section proposes it
// without fixing a confidence score; the one used here is documented in the C
// header).  One thread per row: confident rows keep k_base predictions, the
// others all k_pred; the entries past a row's width become -1 in idx_out.  The
// decision is one fp32 product and one compare, so it is reproducible anywhere.
__global__ __launch_bounds__(SCORE_THREADS) void confidence_select_kernel(
    const int32_t* __restrict__ idx, const float* __restrict__ probs, long long rows, int T, int k_pred, int k_base,
    float ratio, int32_t* __restrict__ idx_out, int32_t* __restrict__ k_row, int32_t* __restrict__ n_wide)
{
    const long long row = (long long)blockIdx.x * SCORE_THREADS + threadIdx.x;
    int wide = 0;
    if (row < rows) {
        const float a = probs[row * k_pred + k_base - 1], b = probs[row * k_pred + k_base];
        const bool confident = a >= __fmul_rn(ratio, b);
        const int w = confident ? k_base : k_pred;
        k_row[row] = w;
        for (int j = 0; j < k_pred; ++j) idx_out[row * k_pred + j] = (j < w) ? idx[row * k_pred + j] : -1;
        wide = !confident;
    }
    // rows of one wave may straddle two layers: count per lane's layer with ballots
    const int layer = (row < rows) ? (int)(row / T) : -1;
    const int first_layer = __shfl(layer, 0, 64);
    const unsigned long long m0 = __ballot(wide && layer == first_layer);
    const unsigned long long m1 = __ballot(wide && layer != first_layer);
    if ((threadIdx.x & 63) == 0 && m0) atomicAdd(&n_wide[first_layer], __popcll(m0));
    if (m1) {                                               // the wave crosses layer boundaries (T < 64): one atomic per row
        if (wide && layer != first_layer) atomicAdd(&n_wide[layer], 1);
    }
}

__global__ void clear_i32_kernel(int32_t* p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

hipError_t launch_confidence_select(const int32_t* idx, const float* probs, int L, int T, int k_pred, int k_base,
                                    float ratio, int32_t* idx_out, int32_t* k_row, int32_t* n_wide,
                                    hipStream_t stream)
{
    hipLaunchKernelGGL(clear_i32_kernel, dim3((L + 255) / 256), dim3(256), 0, stream, n_wide, L);
    const long long rows = (long long)L * T;
    if (rows > 0)
        hipLaunchKernelGGL(confidence_select_kernel, dim3((unsigned)((rows + SCORE_THREADS - 1) / SCORE_THREADS)),
                           dim3(SCORE_THREADS), 0, stream, idx, probs, rows, T, k_pred, k_base, ratio, idx_out, k_row,
                           n_wide);
    return hipGetLastError();
}

}  // namespace paep

// Accuracy counters of the paper's section 5.1: exact match, correctly
// predicted experts, over-provisioning hit, top-1.  One thread per token row
// builds two bitsets over the expert ids (prediction and label), so set
// semantics come for free; rows are reduced per wave with shuffles and added
// to the layer's four 64-bit counters with integer atomics (exact, hence
// deterministic).  A first tiny launch clears the counters.  Short layers take
// a single launch instead: one workgroup per layer, no atomics.
// Rows reach their threads coalesced: a wave reads 64 consecutive rows of a
// [rows][k] array as k loads of 64 consecutive ints (one 256-byte access each;
// a lane reading its own row directly would make every lane a separate access
// to the vector cache, which serves about one access per clock), parks them in
// its own strip of LDS and every lane then picks up its row from there.
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

// raw[j] = element j*64 + lane of a chunk of n_ints consecutive ints (0 past its end): coalesced
template <int KM>
__device__ __forceinline__ void fetch_chunk(const int32_t* __restrict__ g, int k, int n_ints, int lane,
                                            int32_t (&raw)[KM])
{
#pragma unroll
    for (int j = 0; j < KM; ++j) raw[j] = (j < k && j * 64 + lane < n_ints) ? g[j * 64 + lane] : 0;
}

// the chunk goes through the wave's own LDS strip (64 * k ints); lane l comes out with row l of the chunk
template <int KM>
__device__ __forceinline__ void rows_from_chunk(int32_t* strip, int k, int lane, const int32_t (&raw)[KM],
                                                int32_t (&row)[KM])
{
#pragma unroll
    for (int j = 0; j < KM; ++j)
        if (j < k) strip[j * 64 + lane] = raw[j];
    // only this wave uses the strip, and a wave's LDS operations complete in order
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int j = 0; j < KM; ++j) row[j] = (j < k) ? strip[lane * k + j] : 0;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
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

// chunks of 64 rows per wave: four while rows are cheap, one when the kernel is compiled for long rows
template <int KM> struct ScoreChunks { static constexpr int value = (KM <= 8) ? 4 : 1; };

template <int NW, int KM>
__global__ __launch_bounds__(SCORE_THREADS) void score_kernel(
    const int32_t* __restrict__ idx, int k_pred, const int32_t* __restrict__ ref, int k_ref,
    int T, int E, const int32_t* __restrict__ k_row, unsigned long long* __restrict__ counters)
{
    __shared__ int32_t strips[SCORE_THREADS / 64][64 * KM];
    __shared__ int part[SCORE_THREADS / 64][4];
    const int layer = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int v[4] = {0, 0, 0, 0};                                // exact, hits, cover, top1 of this lane's rows (<= 4 * 32 each)
#pragma unroll 1
    for (int c = 0; c < ScoreChunks<KM>::value; ++c) {
        const int t0 = blockIdx.x * (SCORE_THREADS * ScoreChunks<KM>::value) + (c * (SCORE_THREADS / 64) + wave) * 64;   // first row of the chunk
        if (t0 >= T) break;                                 // wave-uniform
        const int rows = (T - t0 < 64) ? T - t0 : 64;
        int32_t rp[KM], rq[KM], pv[KM], qv[KM];
        fetch_chunk<KM>(idx + ((long long)layer * T + t0) * k_pred, k_pred, rows * k_pred, lane, rp);
        fetch_chunk<KM>(ref + ((long long)layer * T + t0) * k_ref, k_ref, rows * k_ref, lane, rq);
        rows_from_chunk<KM>(strips[wave], k_pred, lane, rp, pv);
        rows_from_chunk<KM>(strips[wave], k_ref, lane, rq, qv);
        const int t = t0 + lane;
        if (t < T) {
            const int kp = row_width(k_row, (long long)layer * T + t, k_pred);
            score_vals<NW, KM>(pv, kp, qv, k_ref, E, v[0], v[1], v[2], v[3]);
        }
    }
    // wave reduction, workgroup reduction through LDS, then one atomic per workgroup and counter
    // (64-bit integer atomics: exact, so the order they land in does not matter)
#pragma unroll
    for (int m = 1; m < 64; m <<= 1)
#pragma unroll
        for (int c = 0; c < 4; ++c) v[c] += __shfl_xor(v[c], m, 64);
    if (lane == 0)
#pragma unroll
        for (int c = 0; c < 4; ++c) part[wave][c] = v[c];
    __syncthreads();
    if (threadIdx.x < 4) {
        unsigned long long sum = 0;
        for (int w = 0; w < SCORE_THREADS / 64; ++w) sum += (unsigned long long)part[w][threadIdx.x];
        if (sum) atomicAdd(&counters[(long long)layer * 4 + threadIdx.x], sum);
    }
}

// Up to LAYER_MAX_T tokens per layer: one workgroup per layer walks all rows,
// adds up inside the workgroup and stores the four counters -- one launch, no
// clearing pass and no atomics.
static constexpr int LAYER_MAX_T = 1 << 12;

// waves per workgroup: the LDS strips (64 * KM ints per wave) stay at 32 KB
template <int KM> struct LayerWaves { static constexpr int value = (KM <= 8) ? 16 : (KM <= 16 ? 8 : 4); };

template <int NW, int KM>
__global__ __launch_bounds__(LayerWaves<KM>::value * 64) void score_layer_kernel(
    const int32_t* __restrict__ idx, int k_pred, const int32_t* __restrict__ ref, int k_ref,
    int T, int E, const int32_t* __restrict__ k_row, unsigned long long* __restrict__ counters)
{
    constexpr int WAVES = LayerWaves<KM>::value;
    __shared__ int32_t strips[WAVES][64 * KM];
    __shared__ int part[WAVES][4];
    const int layer = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int v[4] = {0, 0, 0, 0};                                // exact, hits, cover, top1; each < 2^31 (T*k bounded by the caller)
    // a wave takes chunks of 64 rows, RU chunks at a time with all their loads issued before the first is used
    constexpr int RU = (NW > 4) ? 1 : (KM <= 8 ? 4 : (KM <= 16 ? 2 : 1));
    const int32_t* pl = idx + (long long)layer * T * k_pred;
    const int32_t* ql = ref + (long long)layer * T * k_ref;
    for (int c0 = wave; c0 * 64 < T; c0 += WAVES * RU) {
        int32_t rp[RU][KM], rq[RU][KM];
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            const int t0 = (c0 + u * WAVES) * 64;
            if (t0 < T) {                                   // wave-uniform
                const int rows = (T - t0 < 64) ? T - t0 : 64;
                fetch_chunk<KM>(pl + (long long)t0 * k_pred, k_pred, rows * k_pred, lane, rp[u]);
                fetch_chunk<KM>(ql + (long long)t0 * k_ref, k_ref, rows * k_ref, lane, rq[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            const int t0 = (c0 + u * WAVES) * 64;
            if (t0 < T) {
                int32_t pv[KM], qv[KM];
                rows_from_chunk<KM>(strips[wave], k_pred, lane, rp[u], pv);
                rows_from_chunk<KM>(strips[wave], k_ref, lane, rq[u], qv);
                const int t = t0 + lane;
                if (t < T) {
                    const int kp = row_width(k_row, (long long)layer * T + t, k_pred);
                    score_vals<NW, KM>(pv, kp, qv, k_ref, E, v[0], v[1], v[2], v[3]);
                }
            }
        }
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
        for (int w = 0; w < WAVES; ++w) sum += (unsigned long long)part[w][tid];
        counters[(long long)layer * 4 + tid] = sum;
    }
}

template <int NW, int KM>
static void launch_score_cfg(const int32_t* idx, int k_pred, const int32_t* ref, int k_ref, int L, int T, int E,
                             const int32_t* k_row, unsigned long long* c, hipStream_t stream)
{
    // one workgroup per layer while that workgroup's instruction count stays small: it grows with the rows
    // and with the ids per row the kernel is compiled for
    if ((long long)T * KM <= (long long)LAYER_MAX_T * 8) {
        hipLaunchKernelGGL((score_layer_kernel<NW, KM>), dim3(L), dim3(LayerWaves<KM>::value * 64), 0, stream, idx,
                           k_pred, ref, k_ref, T, E, k_row, c);
        return;
    }
    hipLaunchKernelGGL(score_clear_kernel, dim3((4 * L + 255) / 256), dim3(256), 0, stream, c, 4 * L);
    constexpr int ROWS_PER_WG = SCORE_THREADS * ScoreChunks<KM>::value;
    dim3 grid((T + ROWS_PER_WG - 1) / ROWS_PER_WG, L);
    hipLaunchKernelGGL((score_kernel<NW, KM>), grid, dim3(SCORE_THREADS), 0, stream, idx, k_pred, ref, k_ref, T, E,
                       k_row, c);
}

hipError_t launch_score(const int32_t* idx, int k_pred, const int32_t* ref, int k_ref,
                        int L, int T, int E, const int32_t* k_row, long long* counters, hipStream_t stream)
{
    unsigned long long* c = (unsigned long long*)counters;
    // ids per row the kernel is compiled for (the interface allows up to 32)
    const int km = (k_pred <= 8 && k_ref <= 8) ? 8 : ((k_pred <= 16 && k_ref <= 16) ? 16 : 32);
#define PAEP_SCORE_NW(NWV)                                                                          \
    do {                                                                                            \
        if (km == 8)       launch_score_cfg<NWV, 8>(idx, k_pred, ref, k_ref, L, T, E, k_row, c, stream);  \
        else if (km == 16) launch_score_cfg<NWV, 16>(idx, k_pred, ref, k_ref, L, T, E, k_row, c, stream); \
        else               launch_score_cfg<NWV, 32>(idx, k_pred, ref, k_ref, L, T, E, k_row, c, stream); \
    } while (0)
    if (E <= 64)       PAEP_SCORE_NW(1);
    else if (E <= 256) PAEP_SCORE_NW(4);
    else               PAEP_SCORE_NW(16);
#undef PAEP_SCORE_NW
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

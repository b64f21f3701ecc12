// Plain vector-arithmetic predictor kernel: any storage dtype, any shape.
//
// One workgroup (4 waves) handles TS = 4 tokens of one layer.  The token rows
// are widened to fp32 in LDS; each wave then produces one hidden unit at a
// time (lanes split the d-long dot product, coalesced over a W1 row, and
// combine with a fixed-order butterfly), the hidden vector stays in LDS, the
// scores are formed the same way, and each wave finishes one token's softmax
// and top-k (paper eq. 3-4, eq. 1).  It is the path for fp32 storage and for
// shapes the matrix-core kernels do not take; it makes no attempt at speed.
#include "paep_device.h"
#include "paep_internal.h"

namespace paep {

static constexpr int TS = 4;           // tokens per workgroup
static constexpr int SIMPLE_THREADS = 256;

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float* p, long long i) { return p[i]; }
};
template <> struct Elem<uint16_t> {
    static __device__ __forceinline__ float load(const uint16_t* p, long long i) { return bf16_bits_to_f32(p[i]); }
};

template <typename T, bool ROUND_H>
__global__ __launch_bounds__(SIMPLE_THREADS) void predict_simple_kernel(
    int Tn, int d, int r, int E, int k, int act, long long xs, long long w1s, long long w2s,
    const T* __restrict__ x, const T* __restrict__ W1, const T* __restrict__ W2,
    const T* __restrict__ b1, const T* __restrict__ b2,
    int32_t* __restrict__ idx, float* __restrict__ probs, float* __restrict__ logits, int32_t* __restrict__ counts,
    int prob_mode, float* __restrict__ margin)
{
    extern __shared__ float smem[];
    float* xt = smem;                    // [TS][d]
    float* ht = xt + (size_t)TS * d;     // [TS][r]
    float* zt = ht + (size_t)TS * r;     // [TS][E]

    const int layer = blockIdx.y;
    const int t0 = blockIdx.x * TS;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const T* xl = x + (long long)layer * xs;
    const T* W1l = W1 + (long long)layer * w1s;
    const T* W2l = W2 + (long long)layer * w2s;

    for (int i = tid; i < TS * d; i += SIMPLE_THREADS) {
        const int t = i / d, c = i - t * d;
        xt[i] = (t0 + t < Tn) ? Elem<T>::load(xl, (long long)(t0 + t) * d + c) : 0.0f;
    }
    __syncthreads();

    // first linear layer
    for (int j = wave; j < r; j += SIMPLE_THREADS / 64) {
        float acc[TS] = {0.f, 0.f, 0.f, 0.f};
        for (int i = lane; i < d; i += 64) {
            const float w = Elem<T>::load(W1l, (long long)j * d + i);
#pragma unroll
            for (int t = 0; t < TS; ++t) acc[t] = fmaf(w, xt[t * d + i], acc[t]);
        }
#pragma unroll
        for (int t = 0; t < TS; ++t) {
            float v = acc[t];
#pragma unroll
            for (int m = 1; m < 64; m <<= 1) v += __shfl_xor(v, m, 64);
            if (lane == 0) {
                if (b1) v += Elem<T>::load(b1, (long long)layer * r + j);
                if (ROUND_H) v = round_to_bf16(v);
                v = apply_act(v, act);
                if (ROUND_H && act != 0) v = round_to_bf16(v);
                ht[t * r + j] = v;
            }
        }
    }
    __syncthreads();

    // second linear layer
    for (int e = wave; e < E; e += SIMPLE_THREADS / 64) {
        float acc[TS] = {0.f, 0.f, 0.f, 0.f};
        for (int j = lane; j < r; j += 64) {
            const float w = Elem<T>::load(W2l, (long long)e * r + j);
#pragma unroll
            for (int t = 0; t < TS; ++t) acc[t] = fmaf(w, ht[t * r + j], acc[t]);
        }
#pragma unroll
        for (int t = 0; t < TS; ++t) {
            float v = acc[t];
#pragma unroll
            for (int m = 1; m < 64; m <<= 1) v += __shfl_xor(v, m, 64);
            if (lane == 0) {
                if (b2) v += Elem<T>::load(b2, (long long)layer * E + e);
                zt[t * E + e] = v;
                if (logits && t0 + t < Tn) logits[((long long)layer * Tn + t0 + t) * E + e] = v;
            }
        }
    }
    __syncthreads();

    // softmax + top-k: wave w finishes token t0 + w
    const int t = t0 + wave;
    if (t < Tn) {
        const long long row = (long long)layer * Tn + t;
        const EpilogueOut eo{prob_mode, margin ? margin + row : nullptr,
                             counts ? counts + (long long)layer * E : nullptr};
        row_softmax_topk_any<64>(zt + wave * E, E, k, lane, idx + row * k, probs + row * k, eo);
    }
}

static size_t simple_lds_bytes(const PredictArgs& a) { return sizeof(float) * (size_t)TS * ((size_t)a.d + a.r + a.E); }

bool simple_supported(const PredictArgs& a) { return simple_lds_bytes(a) <= 160 * 1024; }

hipError_t launch_predict_simple(const PredictArgs& a)
{
    if (a.T == 0) return hipSuccess;
    const size_t lds = simple_lds_bytes(a);
    dim3 grid((a.T + TS - 1) / TS, a.L);
    hipError_t err;
#define PAEP_LAUNCH_SIMPLE(TY, RH)                                                                   \
    do {                                                                                             \
        auto kern = predict_simple_kernel<TY, RH>;                                                   \
        static LdsLimit limit;                                                                       \
        err = ensure_lds_limit(limit, (const void*)kern, lds);                                       \
        if (err != hipSuccess) return err;                                                           \
        hipLaunchKernelGGL(kern, grid, dim3(SIMPLE_THREADS), lds, a.stream, a.T, a.d, a.r, a.E, a.k, \
                           a.act, a.x_stride, a.w1_stride, a.w2_stride, (const TY*)a.x,              \
                           (const TY*)a.W1, (const TY*)a.W2, (const TY*)a.b1, (const TY*)a.b2,       \
                           a.idx, a.probs, a.logits, a.counts, a.prob_mode, a.margin);               \
    } while (0)
    if (a.dtype == 0) PAEP_LAUNCH_SIMPLE(float, false);
    else              PAEP_LAUNCH_SIMPLE(uint16_t, true);
#undef PAEP_LAUNCH_SIMPLE
    return hipGetLastError();
}

}  // namespace paep

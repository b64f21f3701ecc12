// Decode-shaped predictor (T <= 64 tokens per layer), bf16 storage.
//
// At a handful of tokens the predictor is a weight-streaming problem: every
// byte of W1 (r x d) and W2 (E x r) is needed once and the arithmetic per byte
// is tiny, so the kernel is organised around reading the weights from HBM
// exactly once, coalesced, with many loads in flight.  One predictor belongs
// to one layer (paper section 4.2) and a layer is only ~8 MB, so all layers of
// a call are spread over one grid.
//
// Kernel 1 (partial): the inner width r is cut into slices of RS = 64 hidden
// units; workgroup (slice, layer) owns W1[slice rows, :] and W2[:, slice].
// Wave w streams 16 rows of W1 straight from global memory into the A operand
// of v_mfma_f32_16x16x32_bf16 (each lane reads 16 contiguous bytes of one
// row), the tokens come from a small LDS tile as the B operand (tokens padded
// to a multiple of 16: the matrix cores have throughput to spare here), so the
// slice of the hidden vector h^T[64, T] lands in registers.  It is rounded to
// bf16 (bias and activation applied), parked in LDS, and multiplied by the
// W2 column slice with the same instruction, which gives this slice's
// contribution to the scores; that goes to the workspace as fp32
// partial[layer][slice][t][e].
//
// Kernel 2 (finalize): adds the slices in ascending order (fixed order, so
// the result is reproducible), adds b2, and runs softmax + top-k per token
// (eq. 1 and eq. 4) out of LDS.
#include "paep_device.h"
#include "paep_internal.h"

namespace paep {

static constexpr int DEC_THREADS = 256;
static constexpr int RS = 64;            // hidden units per workgroup (4 waves x 16 rows)
static constexpr int KC = 256;           // d-chunk staged in LDS per step
static constexpr int KSTEPS = KC / 32;   // MFMA k-steps per chunk
static constexpr int XPAD = 8;           // bf16 elements of row padding in LDS
static constexpr int HPAD = 8;

template <int TB>   // 16-token blocks: T <= 16 * TB
__global__ __launch_bounds__(DEC_THREADS) void decode_partial_kernel(
    int T, int d, int r, int E, int act, long long xs_, long long w1s, long long w2s,
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ W1, const uint16_t* __restrict__ W2,
    const uint16_t* __restrict__ b1, float* __restrict__ partial)
{
    constexpr int TP = 16 * TB;
    __shared__ __attribute__((aligned(16))) uint16_t xt[TP * (KC + XPAD)];
    __shared__ __attribute__((aligned(16))) uint16_t ht[TP * (RS + HPAD)];

    const int slice = blockIdx.x, layer = blockIdx.y, S = gridDim.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 15, kg = lane >> 4;
    const uint16_t* xl = x + (long long)layer * xs_;
    const uint16_t* W1l = W1 + (long long)layer * w1s;
    const uint16_t* W2l = W2 + (long long)layer * w2s;

    const int j0 = slice * RS + wave * 16;               // this wave's first hidden unit
    const uint16_t* arow = W1l + (long long)(j0 + m) * d + kg * 8;

    f32x4 acc[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) acc[tb] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int nchunks = d / KC;
    u32x4 a_next[KSTEPS], a_cur[KSTEPS];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) a_next[s] = *(const u32x4*)(arow + s * 32);

    for (int c = 0; c < nchunks; ++c) {
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) a_cur[s] = a_next[s];
        if (c + 1 < nchunks) {
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) a_next[s] = *(const u32x4*)(arow + (c + 1) * KC + s * 32);
        }
        __syncthreads();                                  // previous chunk's LDS reads are done
        for (int i = tid; i < TP * (KC / 8); i += DEC_THREADS) {
            const int t = i / (KC / 8), cv = i - t * (KC / 8);
            u32x4 v = u32x4{0u, 0u, 0u, 0u};
            if (t < T) v = *(const u32x4*)(xl + (long long)t * d + c * KC + cv * 8);
            *(u32x4*)(xt + t * (KC + XPAD) + cv * 8) = v;
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
            const bf16x8 a = __builtin_bit_cast(bf16x8, a_cur[s]);
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                const u32x4 bv = *(const u32x4*)(xt + (tb * 16 + m) * (KC + XPAD) + s * 32 + kg * 8);
                acc[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, bv), acc[tb], 0, 0, 0);
            }
        }
    }

    // acc[tb][i] = h[token tb*16 + m][hidden unit j0 + 4*kg + i]
    float bias[4] = {0.f, 0.f, 0.f, 0.f};
    if (b1) {
#pragma unroll
        for (int i = 0; i < 4; ++i) bias[i] = bf16_bits_to_f32(b1[(long long)layer * r + j0 + 4 * kg + i]);
    }
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float h = round_to_bf16(acc[tb][i] + bias[i]);
            if (act != 0) h = round_to_bf16(apply_act(h, act));
            v[i] = h;
        }
        u32x2 packed = u32x2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
        *(u32x2*)(ht + (tb * 16 + m) * (RS + HPAD) + wave * 16 + 4 * kg) = packed;
    }
    __syncthreads();

    // scores of this slice: z^T[e, t] = W2[e, slice] . h^T[slice, t]
    const int EB = (E + 15) / 16;
    for (int eb = wave; eb < EB; eb += DEC_THREADS / 64) {
        const int e_row = eb * 16 + m;
        u32x4 wfrag[RS / 32];
#pragma unroll
        for (int s = 0; s < RS / 32; ++s) {
            wfrag[s] = u32x4{0u, 0u, 0u, 0u};
            if (e_row < E) wfrag[s] = *(const u32x4*)(W2l + (long long)e_row * r + slice * RS + s * 32 + kg * 8);
        }
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            f32x4 z = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < RS / 32; ++s) {
                const u32x4 hv = *(const u32x4*)(ht + (tb * 16 + m) * (RS + HPAD) + s * 32 + kg * 8);
                z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wfrag[s]),
                                                            __builtin_bit_cast(bf16x8, hv), z, 0, 0, 0);
            }
            // z[i] = score contribution for token tb*16 + m, expert eb*16 + 4*kg + i
            const int t = tb * 16 + m;
            if (t < T) {
                float* dst = partial + (((long long)layer * S + slice) * T + t) * E + eb * 16 + 4 * kg;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (eb * 16 + 4 * kg + i < E) dst[i] = z[i];
            }
        }
    }
}

static constexpr int FIN_G = 16;                          // lanes per token row
static constexpr int FIN_ROWS = DEC_THREADS / FIN_G;      // rows per workgroup

__global__ __launch_bounds__(DEC_THREADS) void decode_finalize_kernel(
    int T, int E, int k, int S, int rows_total, const float* __restrict__ partial,
    const uint16_t* __restrict__ b2, int32_t* __restrict__ idx, float* __restrict__ probs,
    float* __restrict__ logits)
{
    extern __shared__ float zs[];                         // [FIN_ROWS][E + 1]
    const int tid = threadIdx.x;
    const int row0 = blockIdx.x * FIN_ROWS;
    const int ZP = E + 1;
    for (int i = tid; i < FIN_ROWS * E; i += DEC_THREADS) {
        const int rr = i / E, e = i - rr * E;
        const int row = row0 + rr;
        if (row < rows_total) {
            const int layer = row / T, t = row - layer * T;
            const float* src = partial + ((long long)layer * S * T + t) * E + e;
            float z = 0.0f;
            for (int s = 0; s < S; ++s) z += src[(long long)s * T * E];
            if (b2) z += bf16_bits_to_f32(b2[(long long)layer * E + e]);
            zs[rr * ZP + e] = z;
            if (logits) logits[(long long)row * E + e] = z;
        }
    }
    __syncthreads();
    const int rr = tid / FIN_G, g = tid % FIN_G;
    const int row = row0 + rr;
    if (row < rows_total)
        row_softmax_topk_any<FIN_G>(zs + rr * ZP, E, k, g, idx + (long long)row * k, probs + (long long)row * k);
}

bool decode_supported(const PredictArgs& a)
{
    return a.dtype == 1 && a.T >= 1 && a.T <= 64 && a.d % KC == 0 && a.r % RS == 0 && a.E <= 512 && a.k <= 32;
}

size_t decode_workspace_bytes(const PredictArgs& a)
{
    return sizeof(float) * (size_t)a.L * (size_t)(a.r / RS) * (size_t)a.T * (size_t)a.E;
}

hipError_t launch_predict_decode(const PredictArgs& a)
{
    const int S = a.r / RS;
    dim3 grid(S, a.L);
    float* partial = (float*)a.workspace;
    const int TB = (a.T + 15) / 16;
#define PAEP_LAUNCH_DEC(TBV)                                                                          \
    hipLaunchKernelGGL(decode_partial_kernel<TBV>, grid, dim3(DEC_THREADS), 0, a.stream, a.T, a.d,    \
                       a.r, a.E, a.act, a.x_stride, a.w1_stride, a.w2_stride, (const uint16_t*)a.x,   \
                       (const uint16_t*)a.W1, (const uint16_t*)a.W2, (const uint16_t*)a.b1, partial)
    switch (TB) {
    case 1: PAEP_LAUNCH_DEC(1); break;
    case 2: PAEP_LAUNCH_DEC(2); break;
    case 3: PAEP_LAUNCH_DEC(3); break;
    default: PAEP_LAUNCH_DEC(4); break;
    }
#undef PAEP_LAUNCH_DEC
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    const int rows = a.L * a.T;
    const size_t lds = sizeof(float) * (size_t)FIN_ROWS * (size_t)(a.E + 1);
    hipLaunchKernelGGL(decode_finalize_kernel, dim3((rows + FIN_ROWS - 1) / FIN_ROWS), dim3(DEC_THREADS), lds,
                       a.stream, a.T, a.E, a.k, S, rows, partial, (const uint16_t*)a.b2, a.idx, a.probs, a.logits);
    return hipGetLastError();
}

}  // namespace paep

// BatchNorm folded into the predictor's first linear layer.
//
// "Architecture 1" of the paper (section 4.3) is Linear -> BatchNorm -> GELU ->
// Dropout -> Linear.  At inference BatchNorm applies, per hidden unit j, the
// fixed affine map y = g_j (u - mean_j) + beta_j with g_j = gamma_j /
// sqrt(var_j + eps) to u = (W1 x + b1)_j, and dropout is the identity.  The
// affine map commutes into the layer: W1'[j,:] = g_j W1[j,:], b1'[j] =
// g_j (b1[j] - mean_j) + beta_j.  One thread per weight, arithmetic in fp32,
// one rounding to the storage type.
#include "paep_device.h"
#include "paep_internal.h"

namespace paep {

static constexpr int FOLD_THREADS = 256;

template <typename T> struct FoldElem;
template <> struct FoldElem<float> {
    static __device__ __forceinline__ float load(const float* p, long long i) { return p[i]; }
    static __device__ __forceinline__ void store(float* p, long long i, float v) { p[i] = v; }
};
template <> struct FoldElem<uint16_t> {
    static __device__ __forceinline__ float load(const uint16_t* p, long long i) { return bf16_bits_to_f32(p[i]); }
    static __device__ __forceinline__ void store(uint16_t* p, long long i, float v) { p[i] = f32_to_bf16_bits(v); }
};

__device__ __forceinline__ float fold_gain(const float* gamma, const float* var, float eps, long long j)
{
    return __fdiv_rn(gamma[j], __fsqrt_rn(__fadd_rn(var[j], eps)));
}

template <typename T>
__global__ __launch_bounds__(FOLD_THREADS) void fold_batchnorm_kernel(
    const T* __restrict__ W1, const T* __restrict__ b1, const float* __restrict__ gamma,
    const float* __restrict__ beta, const float* __restrict__ mean, const float* __restrict__ var, float eps,
    long long rows, int d, T* W1_out, T* b1_out)
{
    // grid.x walks the rows (layer * r + j), grid.y the columns in blocks of FOLD_THREADS
    const long long row = blockIdx.x;
    if (row >= rows) return;
    const float g = fold_gain(gamma, var, eps, row);
    const int c = blockIdx.y * FOLD_THREADS + threadIdx.x;
    if (c < d) FoldElem<T>::store(W1_out, row * d + c, __fmul_rn(g, FoldElem<T>::load(W1, row * d + c)));
    if (blockIdx.y == 0 && threadIdx.x == 0) {
        const float b = b1 ? FoldElem<T>::load(b1, row) : 0.0f;
        FoldElem<T>::store(b1_out, row, __fadd_rn(__fmul_rn(g, __fsub_rn(b, mean[row])), beta[row]));
    }
}

hipError_t launch_fold_batchnorm(const void* W1, const void* b1, const float* gamma, const float* beta,
                                 const float* mean, const float* var, float eps, int L, int r, int d, int dtype,
                                 void* W1_out, void* b1_out, hipStream_t stream)
{
    const long long rows = (long long)L * r;
    dim3 grid((unsigned)rows, (unsigned)((d + FOLD_THREADS - 1) / FOLD_THREADS));
    if (dtype == 0)
        hipLaunchKernelGGL(fold_batchnorm_kernel<float>, grid, dim3(FOLD_THREADS), 0, stream, (const float*)W1,
                           (const float*)b1, gamma, beta, mean, var, eps, rows, d, (float*)W1_out, (float*)b1_out);
    else
        hipLaunchKernelGGL(fold_batchnorm_kernel<uint16_t>, grid, dim3(FOLD_THREADS), 0, stream,
                           (const uint16_t*)W1, (const uint16_t*)b1, gamma, beta, mean, var, eps, rows, d,
                           (uint16_t*)W1_out, (uint16_t*)b1_out);
    return hipGetLastError();
}

}  // namespace paep

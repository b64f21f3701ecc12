// Host-side launcher prototypes shared between the C-ABI layer and the kernel
// translation units.  Every launcher assumes its arguments were validated by
// the C-ABI layer and returns the hipError_t of its launches.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace paep {

struct PredictArgs {
    int T, d, r, E, k, L, dtype, act;
    long long x_stride, w1_stride, w2_stride;   // elements
    const void* x;
    const void* W1;
    const void* W2;
    const void* b1;
    const void* b2;
    int32_t* idx;
    float* probs;
    float* logits;      // nullable
    int32_t* counts;    // nullable: [L][E] activation counts, added to
    int prob_mode;      // 0 softmax over all E, 1 softmax over the k selected, 2 sigmoid
    float* margin;      // nullable: [L][T] last selected score minus the best score left out
    void* workspace;
    hipStream_t stream;
};

// A kernel's dynamic-LDS limit is raised once per (kernel instantiation, device),
// not on every launch: `bytes` remembers what has been granted on each device.
struct LdsLimit {
    std::atomic<int> bytes[16];
};
inline hipError_t ensure_lds_limit(LdsLimit& st, const void* kern, size_t lds)
{
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    const bool tracked = dev >= 0 && dev < 16;
    if (tracked && (int)lds <= st.bytes[dev].load(std::memory_order_relaxed)) return hipSuccess;
    err = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (err == hipSuccess && tracked) st.bytes[dev].store((int)lds, std::memory_order_relaxed);
    return err;
}

// plain vector-ALU kernel, any dtype / shape
bool simple_supported(const PredictArgs& a);
hipError_t launch_predict_simple(const PredictArgs& a);

// bf16 weight-streaming kernel for T <= 64
bool decode_supported(const PredictArgs& a);
size_t decode_workspace_bytes(const PredictArgs& a);
hipError_t launch_predict_decode(const PredictArgs& a);

// bf16 fused matrix-core kernel for large T
bool prefill_supported(const PredictArgs& a);
size_t prefill_workspace_bytes(const PredictArgs& a);
hipError_t launch_predict_prefill(const PredictArgs& a);
// tile configuration id, workgroups per token tile, chunks of r per workgroup (what the launcher will use)
void prefill_plan(const PredictArgs& a, int* cfg, int* groups, int* chunks_per_group);

size_t group_workspace_bytes(int L, int T, int k, int E);
hipError_t launch_group(const int32_t* idx, int L, int T, int k, int E,
                        int32_t* counts, int32_t* offsets, int32_t* token_pos,
                        int32_t* active, int32_t* n_active, int32_t* n_invalid,
                        void* workspace, hipStream_t stream);

hipError_t launch_fold_batchnorm(const void* W1, const void* b1, const float* gamma, const float* beta,
                                 const float* mean, const float* var, float eps, int L, int r, int d, int dtype,
                                 void* W1_out, void* b1_out, hipStream_t stream);

hipError_t launch_activation_profile(const int32_t* counts, int L, int E, int32_t* order, int32_t* n_active,
                                     double* entropy, hipStream_t stream);

// device-ceiling probes
static constexpr int PROBE_READ_GROUPS = 4096;
hipError_t launch_probe_read(const void* src, size_t bytes, void* sink, hipStream_t stream);
hipError_t launch_probe_mfma(int groups, int iters, void* sink, hipStream_t stream);

hipError_t launch_score(const int32_t* idx, int k_pred, const int32_t* ref, int k_ref,
                        int L, int T, int E, const int32_t* k_row, long long* counters, hipStream_t stream);
hipError_t launch_confidence_select(const int32_t* idx, const float* probs, int L, int T, int k_pred, int k_base,
                                    float ratio, int32_t* idx_out, int32_t* k_row, int32_t* n_wide,
                                    hipStream_t stream);

}  // namespace paep

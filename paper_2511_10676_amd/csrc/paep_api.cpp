// C-ABI layer of the library: argument validation (host only, before any HIP
// call), kernel-family selection, workspace sizing, dispatch.  See
// include/paep.h for the contract of every entry point.
#include "../../include/paep.h"

#include "paep_internal.h"

#include <mutex>

// Scratch memory of paep_predict_static: one array per GPU, allocated when the
// code object is loaded and held until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress; the device address it
// yields (per device) is what kernels and launchers are given.
static __device__ __align__(256) unsigned char scratch[PAEP_STATIC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::mutex scratch_mutex;
void* scratch_dev_ptr[MAX_DEVICES];      // device address of `scratch` on each device, once looked up

// Address of the current device's copy of `scratch` (looked up once per device).
hipError_t scratch_for_current_device(void** out)
{
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_dev_ptr[dev]) {
        void* p = nullptr;
        err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (err != hipSuccess) return err;
        if (!p) return hipErrorInvalidSymbol;
        scratch_dev_ptr[dev] = p;
    }
    *out = scratch_dev_ptr[dev];
    return hipSuccess;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

paep_status check_desc(const paep_predict_desc* d)
{
    if (!d) return PAEP_ERR_NULL;
    if (d->prob != PAEP_PROB_SOFTMAX_ALL && d->prob != PAEP_PROB_SOFTMAX_TOPK && d->prob != PAEP_PROB_SIGMOID)
        return PAEP_ERR_DTYPE;
    if (d->dtype != PAEP_F32 && d->dtype != PAEP_BF16) return PAEP_ERR_DTYPE;
    if (d->act != PAEP_ACT_NONE && d->act != PAEP_ACT_SILU && d->act != PAEP_ACT_GELU) return PAEP_ERR_DTYPE;
    if (d->path < PAEP_PATH_AUTO || d->path > PAEP_PATH_PREFILL) return PAEP_ERR_UNSUPPORTED;
    if (d->T < 0 || d->L < 1 || d->d < 8 || d->r < 8 || d->E < 1 || d->E > PAEP_MAX_E) return PAEP_ERR_SHAPE;
    if (d->d % 8 != 0 || d->r % 8 != 0) return PAEP_ERR_SHAPE;
    if (d->k < 1 || d->k > d->E || d->k > PAEP_MAX_K) return PAEP_ERR_K;
    const long long T = d->T, L = d->L;
    if (T * L >= (1ll << 31) || T * d->k >= (1ll << 30) || T * L * d->E >= (1ll << 40)) return PAEP_ERR_SHAPE;
    if (d->x_layer_stride < 0 || d->w1_layer_stride < 0 || d->w2_layer_stride < 0) return PAEP_ERR_SHAPE;
    if (d->x_layer_stride != 0 && d->x_layer_stride < T * d->d) return PAEP_ERR_SHAPE;
    if (d->w1_layer_stride != 0 && d->w1_layer_stride < (long long)d->r * d->d) return PAEP_ERR_SHAPE;
    if (d->w2_layer_stride != 0 && d->w2_layer_stride < (long long)d->E * d->r) return PAEP_ERR_SHAPE;
    if (d->x_layer_stride % 8 || d->w1_layer_stride % 8 || d->w2_layer_stride % 8) return PAEP_ERR_ALIGN;
    return PAEP_OK;
}

paep::PredictArgs to_args(const paep_predict_desc* d)
{
    paep::PredictArgs a{};
    a.T = d->T; a.d = d->d; a.r = d->r; a.E = d->E; a.k = d->k; a.L = d->L;
    a.dtype = d->dtype; a.act = d->act; a.prob_mode = d->prob;
    a.x_stride = d->x_layer_stride; a.w1_stride = d->w1_layer_stride; a.w2_stride = d->w2_layer_stride;
    return a;
}

// PAEP_PATH_* that will run, or 0 when none can
int resolve(const paep_predict_desc* d, const paep::PredictArgs& a)
{
    // an empty call runs nothing; report the family the shape would use at T = 1
    paep::PredictArgs b = a;
    if (b.T == 0) b.T = 1;
    const bool dec = paep::decode_supported(b), pre = paep::prefill_supported(b), sim = paep::simple_supported(b);
    switch (d->path) {
    case PAEP_PATH_SIMPLE: return sim ? PAEP_PATH_SIMPLE : 0;
    case PAEP_PATH_DECODE: return dec ? PAEP_PATH_DECODE : 0;
    case PAEP_PATH_PREFILL: return pre ? PAEP_PATH_PREFILL : 0;
    default:
        if (dec) return PAEP_PATH_DECODE;
        if (pre) return PAEP_PATH_PREFILL;
        return sim ? PAEP_PATH_SIMPLE : 0;
    }
}

}  // namespace

extern "C" {

int paep_version(void) { return 100; }

const char* paep_status_string(paep_status s)
{
    switch (s) {
    case PAEP_OK: return "ok";
    case PAEP_ERR_NULL: return "a required pointer is NULL";
    case PAEP_ERR_SHAPE: return "a size is out of range or violates a divisibility rule";
    case PAEP_ERR_K: return "k is outside 1..min(E, 32)";
    case PAEP_ERR_DTYPE: return "unknown dtype or activation";
    case PAEP_ERR_ALIGN: return "a pointer or stride is not 16-byte aligned";
    case PAEP_ERR_WORKSPACE: return "workspace is NULL, misaligned or too small";
    case PAEP_ERR_HIP: return "the HIP runtime reported an error";
    case PAEP_ERR_UNSUPPORTED: return "the requested kernel family cannot run this shape";
    }
    return "unknown status";
}

int paep_predict_resolve_path(const paep_predict_desc* desc)
{
    if (check_desc(desc) != PAEP_OK) return -1;
    const int p = resolve(desc, to_args(desc));
    return p ? p : -1;
}

size_t paep_predict_workspace_bytes(const paep_predict_desc* desc)
{
    if (check_desc(desc) != PAEP_OK) return 0;
    const paep::PredictArgs a = to_args(desc);
    const int path = resolve(desc, a);
    if (path == PAEP_PATH_DECODE) return paep::decode_workspace_bytes(a);
    if (path == PAEP_PATH_PREFILL) return paep::prefill_workspace_bytes(a);
    return 0;
}

static paep_status predict_common(const paep_predict_desc* desc,
                                  const void* x_dev, const void* W1_dev, const void* W2_dev,
                                  const void* b1_dev, const void* b2_dev,
                                  int32_t* idx_dev, float* probs_dev, float* logits_dev, int32_t* counts_dev,
                                  float* margin_dev,
                                  void* workspace_dev, size_t workspace_bytes, void* stream)
{
    const paep_status st = check_desc(desc);
    if (st != PAEP_OK) return st;
    if (!W1_dev || !W2_dev) return PAEP_ERR_NULL;
    if (desc->T > 0 && (!x_dev || !idx_dev || !probs_dev)) return PAEP_ERR_NULL;
    if (!aligned16(x_dev) || !aligned16(W1_dev) || !aligned16(W2_dev)) return PAEP_ERR_ALIGN;
    paep::PredictArgs a = to_args(desc);
    a.margin = margin_dev;                                   // the families differ in how many candidates they can keep
    const int path = resolve(desc, a);
    if (!path) return PAEP_ERR_UNSUPPORTED;
    const size_t need = (path == PAEP_PATH_DECODE) ? paep::decode_workspace_bytes(a)
                      : (path == PAEP_PATH_PREFILL) ? paep::prefill_workspace_bytes(a) : 0;
    if (need > 0 && (!workspace_dev || !aligned16(workspace_dev) || workspace_bytes < need)) return PAEP_ERR_WORKSPACE;
    if (desc->T == 0) return PAEP_OK;

    a.x = x_dev; a.W1 = W1_dev; a.W2 = W2_dev; a.b1 = b1_dev; a.b2 = b2_dev;
    a.idx = idx_dev; a.probs = probs_dev; a.logits = logits_dev; a.counts = counts_dev;
    a.workspace = workspace_dev;
    a.stream = static_cast<hipStream_t>(stream);
    hipError_t err;
    switch (path) {
    case PAEP_PATH_DECODE: err = paep::launch_predict_decode(a); break;
    case PAEP_PATH_PREFILL: err = paep::launch_predict_prefill(a); break;
    default: err = paep::launch_predict_simple(a); break;
    }
    return err == hipSuccess ? PAEP_OK : PAEP_ERR_HIP;
}

paep_status paep_predict(const paep_predict_desc* desc,
                         const void* x_dev, const void* W1_dev, const void* W2_dev,
                         const void* b1_dev, const void* b2_dev,
                         int32_t* idx_dev, float* probs_dev, float* logits_dev,
                         void* workspace_dev, size_t workspace_bytes, void* stream)
{
    return predict_common(desc, x_dev, W1_dev, W2_dev, b1_dev, b2_dev, idx_dev, probs_dev, logits_dev, nullptr,
                          nullptr, workspace_dev, workspace_bytes, stream);
}

paep_status paep_predict_counted(const paep_predict_desc* desc,
                                 const void* x_dev, const void* W1_dev, const void* W2_dev,
                                 const void* b1_dev, const void* b2_dev,
                                 int32_t* idx_dev, float* probs_dev, float* logits_dev, int32_t* counts_dev,
                                 void* workspace_dev, size_t workspace_bytes, void* stream)
{
    if (!counts_dev) return PAEP_ERR_NULL;
    return predict_common(desc, x_dev, W1_dev, W2_dev, b1_dev, b2_dev, idx_dev, probs_dev, logits_dev, counts_dev,
                          nullptr, workspace_dev, workspace_bytes, stream);
}

paep_status paep_predict_confidence(const paep_predict_desc* desc,
                                    const void* x_dev, const void* W1_dev, const void* W2_dev,
                                    const void* b1_dev, const void* b2_dev,
                                    int32_t* idx_dev, float* probs_dev, float* logits_dev,
                                    int32_t* counts_dev, float* margin_dev,
                                    void* workspace_dev, size_t workspace_bytes, void* stream)
{
    return predict_common(desc, x_dev, W1_dev, W2_dev, b1_dev, b2_dev, idx_dev, probs_dev, logits_dev, counts_dev,
                          margin_dev, workspace_dev, workspace_bytes, stream);
}

paep_status paep_static_init(void)
{
    void* p = nullptr;
    return scratch_for_current_device(&p) == hipSuccess ? PAEP_OK : PAEP_ERR_HIP;
}

paep_status paep_predict_static(const paep_predict_desc* desc,
                                const void* x_dev, const void* W1_dev, const void* W2_dev,
                                const void* b1_dev, const void* b2_dev,
                                int32_t* idx_dev, float* probs_dev, float* logits_dev, void* stream)
{
    const paep_status st = check_desc(desc);
    if (st != PAEP_OK) return st;
    const size_t need = paep_predict_workspace_bytes(desc);
    if (need > (size_t)PAEP_STATIC_SCRATCH_BYTES) return PAEP_ERR_WORKSPACE;
    void* ws = nullptr;
    if (scratch_for_current_device(&ws) != hipSuccess) return PAEP_ERR_HIP;
    return predict_common(desc, x_dev, W1_dev, W2_dev, b1_dev, b2_dev, idx_dev, probs_dev, logits_dev, nullptr,
                          nullptr, ws, (size_t)PAEP_STATIC_SCRATCH_BYTES, stream);
}

paep_status paep_predict_plan(const paep_predict_desc* desc, int32_t want_margin, int32_t plan[4])
{
    const paep_status st = check_desc(desc);
    if (st != PAEP_OK) return st;
    if (!plan) return PAEP_ERR_NULL;
    paep::PredictArgs a = to_args(desc);
    static float margin_wanted;                              // only its address matters: "a margin output is present"
    a.margin = want_margin ? &margin_wanted : nullptr;
    const int path = resolve(desc, a);
    if (!path) return PAEP_ERR_UNSUPPORTED;
    plan[0] = path; plan[1] = 0; plan[2] = 1; plan[3] = 0;
    if (path == PAEP_PATH_PREFILL) {
        if (a.T == 0) a.T = 1;
        int cfg = 0, groups = 1, cpg = 0;
        paep::prefill_plan(a, &cfg, &groups, &cpg);
        plan[1] = cfg; plan[2] = groups; plan[3] = cpg;
    }
    return PAEP_OK;
}

paep_status paep_fold_batchnorm(const void* W1_dev, const void* b1_dev, const float* gamma_dev,
                                const float* beta_dev, const float* mean_dev, const float* var_dev, float eps,
                                int32_t L, int32_t r, int32_t d, int32_t dtype, void* W1_out_dev,
                                void* b1_out_dev, void* stream)
{
    if (L < 1 || r < 1 || d < 1 || (long long)L * r >= (1ll << 31) || (long long)L * r * d >= (1ll << 40))
        return PAEP_ERR_SHAPE;
    if (dtype != PAEP_F32 && dtype != PAEP_BF16) return PAEP_ERR_DTYPE;
    if (!(eps >= 0.0f)) return PAEP_ERR_SHAPE;               // also rejects NaN
    if (!W1_dev || !gamma_dev || !beta_dev || !mean_dev || !var_dev || !W1_out_dev || !b1_out_dev)
        return PAEP_ERR_NULL;
    const hipError_t err = paep::launch_fold_batchnorm(W1_dev, b1_dev, gamma_dev, beta_dev, mean_dev, var_dev, eps,
                                                       L, r, d, dtype, W1_out_dev, b1_out_dev,
                                                       static_cast<hipStream_t>(stream));
    return err == hipSuccess ? PAEP_OK : PAEP_ERR_HIP;
}

static paep_status check_group(int32_t L, int32_t T, int32_t k, int32_t E)
{
    if (L < 1 || T < 0 || E < 1 || E > PAEP_MAX_E) return PAEP_ERR_SHAPE;
    if (k < 1 || k > PAEP_MAX_K) return PAEP_ERR_K;
    if ((long long)T * k >= (1ll << 30) || (long long)T * k * L >= (1ll << 40)) return PAEP_ERR_SHAPE;
    return PAEP_OK;
}

size_t paep_group_workspace_bytes(int32_t L, int32_t T, int32_t k, int32_t E)
{
    if (check_group(L, T, k, E) != PAEP_OK) return 0;
    return paep::group_workspace_bytes(L, T, k, E);
}

paep_status paep_group_by_expert(const int32_t* idx_dev, int32_t L, int32_t T, int32_t k, int32_t E,
                                 int32_t* counts_dev, int32_t* offsets_dev, int32_t* token_pos_dev,
                                 int32_t* active_dev, int32_t* n_active_dev, int32_t* n_invalid_dev,
                                 void* workspace_dev, size_t workspace_bytes, void* stream)
{
    const paep_status st = check_group(L, T, k, E);
    if (st != PAEP_OK) return st;
    if (!counts_dev || !offsets_dev || !active_dev || !n_active_dev || !n_invalid_dev) return PAEP_ERR_NULL;
    if (T > 0 && (!idx_dev || !token_pos_dev)) return PAEP_ERR_NULL;
    const size_t need = paep::group_workspace_bytes(L, T, k, E);
    if (need > 0 && (!workspace_dev || !aligned16(workspace_dev) || workspace_bytes < need)) return PAEP_ERR_WORKSPACE;
    const hipError_t err = paep::launch_group(idx_dev, L, T, k, E, counts_dev, offsets_dev, token_pos_dev,
                                              active_dev, n_active_dev, n_invalid_dev, workspace_dev,
                                              static_cast<hipStream_t>(stream));
    return err == hipSuccess ? PAEP_OK : PAEP_ERR_HIP;
}

static paep_status score_common(const int32_t* idx_dev, int32_t k_pred, const int32_t* k_row_dev,
                                const int32_t* ref_dev, int32_t k_ref, int32_t L, int32_t T, int32_t E,
                                long long* counters_dev, void* stream)
{
    if (L < 1 || T < 0 || E < 1 || E > PAEP_MAX_E) return PAEP_ERR_SHAPE;
    if (k_pred < 1 || k_pred > PAEP_MAX_K || k_ref < 1 || k_ref > PAEP_MAX_K) return PAEP_ERR_K;
    if ((long long)T * L >= (1ll << 31)) return PAEP_ERR_SHAPE;
    if (!counters_dev) return PAEP_ERR_NULL;
    if (T > 0 && (!idx_dev || !ref_dev)) return PAEP_ERR_NULL;
    const hipError_t err = paep::launch_score(idx_dev, k_pred, ref_dev, k_ref, L, T, E, k_row_dev, counters_dev,
                                              static_cast<hipStream_t>(stream));
    return err == hipSuccess ? PAEP_OK : PAEP_ERR_HIP;
}

paep_status paep_score(const int32_t* idx_dev, int32_t k_pred, const int32_t* ref_dev, int32_t k_ref,
                       int32_t L, int32_t T, int32_t E, long long* counters_dev, void* stream)
{
    return score_common(idx_dev, k_pred, nullptr, ref_dev, k_ref, L, T, E, counters_dev, stream);
}

paep_status paep_score_rows(const int32_t* idx_dev, int32_t k_pred, const int32_t* k_row_dev,
                            const int32_t* ref_dev, int32_t k_ref, int32_t L, int32_t T, int32_t E,
                            long long* counters_dev, void* stream)
{
    if (T > 0 && !k_row_dev) return PAEP_ERR_NULL;
    return score_common(idx_dev, k_pred, k_row_dev, ref_dev, k_ref, L, T, E, counters_dev, stream);
}

paep_status paep_confidence_select(const int32_t* idx_dev, const float* probs_dev, int32_t L, int32_t T,
                                   int32_t k_pred, int32_t k_base, float ratio, int32_t* idx_out_dev,
                                   int32_t* k_row_dev, int32_t* n_wide_dev, void* stream)
{
    if (L < 1 || T < 0 || (long long)T * L >= (1ll << 31)) return PAEP_ERR_SHAPE;
    if (k_pred < 2 || k_pred > PAEP_MAX_K || k_base < 1 || k_base >= k_pred) return PAEP_ERR_K;
    if (!(ratio >= 1.0f)) return PAEP_ERR_SHAPE;             // also rejects NaN
    if (!n_wide_dev) return PAEP_ERR_NULL;
    if (T > 0 && (!idx_dev || !probs_dev || !idx_out_dev || !k_row_dev)) return PAEP_ERR_NULL;
    const hipError_t err = paep::launch_confidence_select(idx_dev, probs_dev, L, T, k_pred, k_base, ratio,
                                                          idx_out_dev, k_row_dev, n_wide_dev,
                                                          static_cast<hipStream_t>(stream));
    return err == hipSuccess ? PAEP_OK : PAEP_ERR_HIP;
}

paep_status paep_activation_profile(const int32_t* counts_dev, int32_t L, int32_t E, int32_t* order_dev,
                                    int32_t* n_active_dev, double* entropy_dev, void* stream)
{
    if (L < 1 || E < 1 || E > PAEP_MAX_E) return PAEP_ERR_SHAPE;
    if (!counts_dev || !order_dev || !n_active_dev || !entropy_dev) return PAEP_ERR_NULL;
    const hipError_t err = paep::launch_activation_profile(counts_dev, L, E, order_dev, n_active_dev, entropy_dev,
                                                           static_cast<hipStream_t>(stream));
    return err == hipSuccess ? PAEP_OK : PAEP_ERR_HIP;
}

paep_status paep_probe_read(const void* src_dev, size_t bytes, void* sink_dev, size_t sink_bytes, void* stream)
{
    if (!src_dev || !sink_dev) return PAEP_ERR_NULL;
    if (bytes % 16 != 0 || (reinterpret_cast<uintptr_t>(src_dev) & 15u)) return PAEP_ERR_ALIGN;
    if (sink_bytes < 16u * paep::PROBE_READ_GROUPS) return PAEP_ERR_WORKSPACE;
    const hipError_t err = paep::launch_probe_read(src_dev, bytes, sink_dev, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? PAEP_OK : PAEP_ERR_HIP;
}

paep_status paep_probe_mfma(int32_t workgroups, int32_t iters, void* sink_dev, size_t sink_bytes, void* stream,
                            double* flops_out)
{
    if (workgroups < 1 || workgroups > 65536 || iters < 1) return PAEP_ERR_SHAPE;
    if (!sink_dev) return PAEP_ERR_NULL;
    if (sink_bytes < 4u * (size_t)workgroups) return PAEP_ERR_WORKSPACE;
    // 8 waves per workgroup, 8 instructions per iteration, 2*32*32*16 flops each
    if (flops_out) *flops_out = (double)workgroups * 8.0 * (double)iters * 8.0 * 32768.0;
    const hipError_t err = paep::launch_probe_mfma(workgroups, iters, sink_dev, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? PAEP_OK : PAEP_ERR_HIP;
}

}  // extern "C"

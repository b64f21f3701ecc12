/*
 * paep -- pre-attention expert prediction for Mixture-of-Experts models,
 * C ABI of the MI355X (gfx950) library.
 *
 * The paper ("Pre-Attention Expert Prediction and Prefetching for
 * Mixture-of-Experts Large Language Models") attaches to every MoE layer a
 * small predictor that reads the hidden state X entering the layer's attention
 * block and names the experts the layer's router will pick, so that they can
 * be prefetched while attention runs (sections 4.1-4.2).  This library is the
 * data-parallel part of that: the predictor itself for many tokens and layers
 * at once, the per-expert grouping of its selections (the prefetch list), and
 * the accuracy counters of section 5.1.
 *
 * Conventions for every entry point
 *   - Pointers named *_dev are DEVICE pointers owned by the caller (inputs,
 *     outputs and workspace alike); the library allocates nothing, frees
 *     nothing and keeps no pointer after it returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All work is enqueued on it; nothing synchronises.  Outputs are valid
 *     once the caller has synchronised the stream.
 *   - All arrays are dense, row-major, with the strides stated.
 *   - Every argument check runs on the host before the first HIP call and
 *     returns a status code; no entry point throws, aborts or prints.
 *     A failed launch returns PAEP_ERR_HIP.
 *   - Results are deterministic: the same inputs give the same bytes.
 *   - Zero tokens (T = 0) is valid and produces empty / all-zero outputs.
 */
#ifndef PAEP_H
#define PAEP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PAEP_OK = 0,
    PAEP_ERR_NULL = 1,        /* a required pointer is NULL */
    PAEP_ERR_SHAPE = 2,       /* a size is out of range or violates a divisibility rule */
    PAEP_ERR_K = 3,           /* k outside 1..min(E, PAEP_MAX_K) */
    PAEP_ERR_DTYPE = 4,       /* unknown dtype or activation */
    PAEP_ERR_ALIGN = 5,       /* a pointer or stride breaks the 16-byte alignment rule */
    PAEP_ERR_WORKSPACE = 6,   /* workspace NULL or smaller than the *_workspace_bytes answer */
    PAEP_ERR_HIP = 7,         /* the HIP runtime reported an error */
    PAEP_ERR_UNSUPPORTED = 8  /* the forced path cannot run this shape */
} paep_status;

typedef enum { PAEP_F32 = 0, PAEP_BF16 = 1 } paep_dtype;

/* Element-wise function between the two linear layers (section 4.3):
 * NONE is the plain two-linear predictor of the abstract and section 1,
 * SILU is "Architecture 2", GELU (exact, erf) is "Architecture 1" at
 * inference time with its BatchNorm folded into W1 and b1 by the caller. */
typedef enum { PAEP_ACT_NONE = 0, PAEP_ACT_SILU = 1, PAEP_ACT_GELU = 2 } paep_act;

/* Kernel family.  AUTO picks by shape; the others force one and fail with
 * PAEP_ERR_UNSUPPORTED when the shape does not fit it. */
typedef enum {
    PAEP_PATH_AUTO = 0,
    PAEP_PATH_SIMPLE = 1,     /* any dtype and shape; plain vector arithmetic */
    PAEP_PATH_DECODE = 2,     /* bf16, T <= 64: weight-streaming, r split over workgroups */
    PAEP_PATH_PREFILL = 3     /* bf16, large T: fused back-to-back matrix-core tiles */
} paep_path;

/* What paep_predict writes to probs for the selected experts.  The paper's
 * predictor is trained through a sigmoid (binary cross-entropy per expert,
 * section 4.4) while the router it imitates normalises with a softmax (eq. 1);
 * its closing section asks for per-prediction confidence scores.  All three
 * are monotone in the score, so the selection is the same.
 *   SOFTMAX_ALL   softmax over all E scores, gathered at the selection
 *   SOFTMAX_TOPK  softmax over the k selected scores only (sums to 1 per row)
 *   SIGMOID       1 / (1 + exp(-s)) of each selected score                    */
typedef enum { PAEP_PROB_SOFTMAX_ALL = 0, PAEP_PROB_SOFTMAX_TOPK = 1, PAEP_PROB_SIGMOID = 2 } paep_prob;

#define PAEP_MAX_K 32
#define PAEP_MAX_E 1024

/*
 * Shape of one predict call.  L layers are processed in one call; layer l
 * reads x + l*x_layer_stride, W1 + l*w1_layer_stride, W2 + l*w2_layer_stride
 * (strides in ELEMENTS; x_layer_stride = 0 feeds the same tokens to every
 * layer; the weight strides must be >= the matrix size, or 0 to share).
 */
typedef struct {
    int32_t T;          /* tokens per layer, >= 0 */
    int32_t d;          /* hidden size, multiple of 8 */
    int32_t r;          /* predictor inner width, multiple of 8 */
    int32_t E;          /* experts, 1..PAEP_MAX_E */
    int32_t k;          /* experts to select, 1..min(E, PAEP_MAX_K) */
    int32_t L;          /* layers in this call, >= 1 */
    int32_t dtype;      /* paep_dtype of x, W1, W2, b1, b2 */
    int32_t act;        /* paep_act */
    int32_t path;       /* paep_path */
    int32_t prob;       /* paep_prob; 0 = softmax over all E */
    int64_t x_layer_stride;
    int64_t w1_layer_stride;
    int64_t w2_layer_stride;
} paep_predict_desc;

/* Bytes of device workspace paep_predict needs for this shape (0 is possible).
 * Returns 0 for an invalid descriptor; paep_predict reports the reason. */
size_t paep_predict_workspace_bytes(const paep_predict_desc *desc);

/* Which kernel family AUTO resolves to for this shape (a paep_path value),
 * or -1 for an invalid descriptor.  Host only. */
int paep_predict_resolve_path(const paep_predict_desc *desc);

/*
 * The predictor (paper eq. 3-4 with f = two linear layers, section 4.3;
 * softmax as in eq. 1).  For every layer l and token t:
 *     h = W1_l x_t (+ b1_l);   in bf16 storage h is rounded to bf16;  h = act(h)
 *     s = W2_l h   (+ b2_l)                      scores, fp32
 *     idx[l,t,:]   = the k experts with the highest s, in descending score
 *                    order, equal scores by ascending expert id
 *     probs[l,t,j] = softmax(s)[idx[l,t,j]]      over all E scores (desc->prob = 0;
 *                    see paep_prob for the other two confidence scores)
 * Selection is done on the raw scores: softmax preserves ranking
 * (sections 1 and 3.1).  h and s never go to memory unless logits_dev is
 * given.
 *
 *   x_dev   [L or 1][T, d]   W1_dev [L][r, d]   W2_dev [L][E, r]
 *   b1_dev  [L][r] or NULL   b2_dev [L][E] or NULL   (dense, layer stride r / E)
 *   idx_dev [L][T, k] int32  probs_dev [L][T, k] float
 *   logits_dev [L][T, E] float or NULL: the scores s, for checking only
 *   workspace_dev: at least paep_predict_workspace_bytes(desc) bytes,
 *                  16-byte aligned; may be NULL when that is 0.  Contents on
 *                  entry do not matter; calls that may run at the same time
 *                  (different streams) need a workspace each.
 * x, W1, W2 and their layer strides must be 16-byte aligned.  With T = 0 the
 * token-sized arrays (x, idx, probs, logits) may be NULL.
 * Inputs must be finite; a NaN score orders below every number.
 */
paep_status paep_predict(const paep_predict_desc *desc,
                         const void *x_dev, const void *W1_dev, const void *W2_dev,
                         const void *b1_dev, const void *b2_dev,
                         int32_t *idx_dev, float *probs_dev, float *logits_dev,
                         void *workspace_dev, size_t workspace_bytes, void *stream);

/*
 * paep_predict that also counts the selections: counts_dev[l][e] (int32,
 * [L][E], required) is INCREASED by the number of tokens of layer l whose
 * selection contains expert e -- the histogram paep_group_by_expert would
 * compute, produced in the predictor's epilogue with integer atomics (exact,
 * order-independent).  The caller zeroes counts_dev when a fresh histogram is
 * wanted, or leaves it to accumulate expert popularity over calls, e.g. over
 * the decode steps of a generation (the activation frequencies of section 2.1);
 * paep_activation_profile turns it into a popularity order.  Everything else
 * as in paep_predict.
 */
paep_status paep_predict_counted(const paep_predict_desc *desc,
                                 const void *x_dev, const void *W1_dev, const void *W2_dev,
                                 const void *b1_dev, const void *b2_dev,
                                 int32_t *idx_dev, float *probs_dev, float *logits_dev, int32_t *counts_dev,
                                 void *workspace_dev, size_t workspace_bytes, void *stream);

/*
 * paep_predict with the confidence outputs the paper's closing section asks
 * for (prediction confidence scores that drive dynamic over-provisioning):
 *   margin_dev [L][T] float, nullable: for every row, the score of the last
 *       selected expert minus the best score that was left out,
 *       s(k-th) - s((k+1)-th) >= 0; +infinity when k = E.  A small margin
 *       marks a row whose selection a small error could change.
 *   counts_dev as in paep_predict_counted, nullable here.
 * probs follows desc->prob as in every predict call.  With the margin the
 * kernels keep one more candidate per row, so k <= PAEP_MAX_K still holds but
 * the matrix-core prefill path takes k <= 15 (k <= 16 without).
 */
paep_status paep_predict_confidence(const paep_predict_desc *desc,
                                    const void *x_dev, const void *W1_dev, const void *W2_dev,
                                    const void *b1_dev, const void *b2_dev,
                                    int32_t *idx_dev, float *probs_dev, float *logits_dev,
                                    int32_t *counts_dev, float *margin_dev,
                                    void *workspace_dev, size_t workspace_bytes, void *stream);

/*
 * paep_predict for callers that cannot allocate device memory or carry a
 * workspace around: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same computation, same kernels and same
 * results as paep_predict; the workspace is a buffer of
 * PAEP_STATIC_SCRATCH_BYTES that lives inside the library's code object, one
 * copy per GPU, held until the process ends.  The call allocates and frees
 * nothing (no hipMalloc, no hipFree, no allocating library routine).
 *   - Shapes whose paep_predict_workspace_bytes exceeds
 *     PAEP_STATIC_SCRATCH_BYTES return PAEP_ERR_WORKSPACE (16 MiB covers the
 *     decode path of a DeepSeek-V2-Lite-sized bank up to 64 tokens and every
 *     prefill shape that needs no r split); nothing is launched then.
 *   - Every call on a GPU uses that GPU's one buffer, which keeps whatever the
 *     last call left in it; the kernels overwrite (or clear with a fill kernel)
 *     every part they later read.  Two calls that may overlap on one GPU
 *     (different streams, or several host threads) race on it: serialise them,
 *     or use paep_predict with a workspace each.
 *   - The first call on a device looks up the device address of the buffer
 *     (hipGetSymbolAddress).  paep_static_init() does that ahead of time for
 *     the current device -- call it once per device before capturing a graph.
 */
#define PAEP_STATIC_SCRATCH_BYTES (16u << 20)
paep_status paep_static_init(void);
paep_status paep_predict_static(const paep_predict_desc *desc,
                                const void *x_dev, const void *W1_dev, const void *W2_dev,
                                const void *b1_dev, const void *b2_dev,
                                int32_t *idx_dev, float *probs_dev, float *logits_dev, void *stream);

/*
 * How paep_predict (want_margin = 0) or paep_predict_confidence with a margin
 * output (want_margin = 1) will run this shape.  Host only; for tests and reports.
 *   plan[0] kernel family (paep_path)
 *   plan[1] tile configuration of the prefill family (0 otherwise):
 *           0 128x128, 1 128x128 wide, 2 256x256, 3 256x128, 4 256x256 wide
 *   plan[2] workgroups that share one token tile (the inner width r split
 *           between them; 1 = no split, no workspace)
 *   plan[3] chunks of r each of them walks
 * Returns PAEP_OK, or the status paep_predict would give for the descriptor.
 */
paep_status paep_predict_plan(const paep_predict_desc *desc, int32_t want_margin, int32_t plan[4]);

/*
 * Architecture 1 of section 4.3 puts BatchNorm between the first linear layer
 * and GELU.  At inference BatchNorm is the affine map
 *     y_j = gamma_j (u_j - mean_j) / sqrt(var_j + eps) + beta_j
 * on u = W1 x + b1, so it folds into the first layer:
 *     W1'[j,:] = g_j W1[j,:],   b1'[j] = g_j (b1[j] - mean_j) + beta_j,   g_j = gamma_j / sqrt(var_j + eps)
 * and paep_predict with act = GELU on (W1', b1') is the whole block (dropout
 * is the identity at inference).  This call computes W1' and b1' on the
 * device, in fp32, rounded once to the storage dtype.
 *   W1_dev [L][r,d], b1_dev [L][r] or NULL (= 0) in `dtype`;
 *   gamma/beta/mean/var_dev [L][r] float;  W1_out_dev [L][r,d], b1_out_dev [L][r] in `dtype`
 *   (W1_out_dev may be W1_dev: in place).  var + eps must be > 0.
 */
paep_status paep_fold_batchnorm(const void *W1_dev, const void *b1_dev,
                                const float *gamma_dev, const float *beta_dev,
                                const float *mean_dev, const float *var_dev, float eps,
                                int32_t L, int32_t r, int32_t d, int32_t dtype,
                                void *W1_out_dev, void *b1_out_dev, void *stream);

/* Workspace bytes for paep_group_by_expert (0 when the single-launch path
 * serves the shape). */
size_t paep_group_workspace_bytes(int32_t L, int32_t T, int32_t k, int32_t E);

/*
 * Per-expert grouping of the selections, i.e. the prefetch list of the paper's
 * workflow (section 4.2, third stage: the selected experts drive prefetching).
 * For every layer l, over the n = T*k flat positions p = t*k + j of idx[l]:
 *     counts[l,e]     number of positions with idx = e
 *     offsets[l,0..E] exclusive prefix sum of counts; offsets[l,E] = number
 *                     of valid positions
 *     token_pos[l, offsets[l,e] .. offsets[l,e+1]) = the positions p with
 *                     idx = e in ascending p (token = p / k, slot = p % k);
 *                     entries past offsets[l,E] are -1
 *     active[l, 0..n_active[l]) = the experts with counts > 0, ascending id
 *                     (the experts to prefetch); the rest of the row is -1
 *     n_invalid[l]    positions whose id is outside [0, E): they are skipped
 * All outputs int32.  Requires T*k < 2^31 / 2 and E <= PAEP_MAX_E.
 * workspace_dev: at least paep_group_workspace_bytes(L, T, k, E) bytes, 16-byte
 * aligned; may be NULL when that is 0.
 */
paep_status paep_group_by_expert(const int32_t *idx_dev, int32_t L, int32_t T, int32_t k, int32_t E,
                                 int32_t *counts_dev, int32_t *offsets_dev, int32_t *token_pos_dev,
                                 int32_t *active_dev, int32_t *n_active_dev, int32_t *n_invalid_dev,
                                 void *workspace_dev, size_t workspace_bytes, void *stream);

/*
 * Accuracy counters of section 5.1 (and the deployment scenarios at the end
 * of section 4.1).  For every layer l and token t let P = set(idx[l,t,:k_pred])
 * and R = set(ref[l,t,:k_ref]); then
 *     counters[l,0] += (P == R)          exact match
 *     counters[l,1] += |P & R|           correctly predicted experts
 *     counters[l,2] += (R subset of P)   hit under over-provisioning (k_pred > k_ref)
 *     counters[l,3] += (idx[l,t,0] in R) top-1
 * A row holding an id outside [0, E) in either array adds nothing.
 * counters_dev is [L, 4] int64 and is overwritten (not accumulated into).
 */
paep_status paep_score(const int32_t *idx_dev, int32_t k_pred,
                       const int32_t *ref_dev, int32_t k_ref,
                       int32_t L, int32_t T, int32_t E,
                       long long *counters_dev, void *stream);

/*
 * paep_score with a width per row: row (l, t) uses only its first
 * clamp(k_row[l,t], 1, k_pred) predicted ids; ids past that width are not
 * looked at (so the -1 padding paep_confidence_select writes is fine).
 * k_row_dev is [L][T] int32.  Everything else as in paep_score.
 */
paep_status paep_score_rows(const int32_t *idx_dev, int32_t k_pred, const int32_t *k_row_dev,
                            const int32_t *ref_dev, int32_t k_ref,
                            int32_t L, int32_t T, int32_t E,
                            long long *counters_dev, void *stream);

/*
 * Confidence-driven over-provisioning, the extension the paper's closing
 * section sketches: rows predicted with high confidence are served in
 * exact-match mode (k_base experts), the others are over-provisioned (all
 * k_pred experts that paep_predict returned).  The paper fixes no confidence
 * score; this one is the separation between the last expert inside the
 * exact-match set and the first one outside it.  Row (l, t) is confident when
 *     probs[l,t,k_base-1] >= ratio * probs[l,t,k_base]        (in float)
 * i.e. ratio = exp(tau) asks for a margin tau between the two scores, because
 * the softmax of one row shares one normaliser.  ratio >= 1.
 *     k_row[l,t]      = k_base if confident, else k_pred
 *     idx_out[l,t,j]  = idx[l,t,j] for j < k_row[l,t], else -1
 *                       (paep_group_by_expert skips the -1 entries and counts
 *                       them in n_invalid; idx_out must not overlap idx)
 *     n_wide[l]       = number of rows of layer l that were widened
 * idx_dev, idx_out_dev [L][T, k_pred] int32; probs_dev [L][T, k_pred] float as
 * written by paep_predict (descending); k_row_dev [L][T] int32; n_wide_dev [L]
 * int32.  1 <= k_base < k_pred <= PAEP_MAX_K.
 */
paep_status paep_confidence_select(const int32_t *idx_dev, const float *probs_dev,
                                   int32_t L, int32_t T, int32_t k_pred, int32_t k_base, float ratio,
                                   int32_t *idx_out_dev, int32_t *k_row_dev, int32_t *n_wide_dev, void *stream);

/*
 * Expert popularity per layer from the activation counts that
 * paep_group_by_expert produced (section 2.1: distribution of expert
 * activation frequencies and its Shannon entropy; section 2.2.2: prefetching
 * by expert popularity).  For every layer l:
 *     order[l, 0..n_active[l]) = the experts with counts > 0 by descending
 *                     count, equal counts by ascending id; the rest is -1
 *     entropy[l]    = -sum_e p_e ln p_e / ln E,  p_e = counts[l,e] / sum_e counts[l,e],
 *                     in double; 0 when E = 1 or the layer counted nothing
 * counts_dev [L][E] int32 (negative entries count as 0), order_dev [L][E]
 * int32, n_active_dev [L] int32, entropy_dev [L] double.  E <= PAEP_MAX_E.
 */
paep_status paep_activation_profile(const int32_t *counts_dev, int32_t L, int32_t E, int32_t *order_dev,
                                    int32_t *n_active_dev, double *entropy_dev, void *stream);

/*
 * Device ceilings, measured: not part of the paper's method.  The benchmark
 * runs them next to the predict kernels so that a roofline fraction can be
 * read against what this device sustains as well as against the published peak.
 *
 * paep_probe_read: one launch that reads `bytes` (multiple of 16, 16-byte
 *   aligned) from src_dev with coalesced 16-byte loads and folds them into
 *   sink_dev (at least 65536 bytes; contents are meaningless).
 * paep_probe_mfma: one launch of `workgroups` workgroups of eight waves, each
 *   issuing 8 * iters v_mfma_f32_32x32x16_bf16 from registers; *flops_out
 *   (host, may be NULL) receives the flops of the launch; sink_dev needs 4
 *   bytes per workgroup.
 * Both are asynchronous on `stream`; time them with events.
 */
paep_status paep_probe_read(const void *src_dev, size_t bytes, void *sink_dev, size_t sink_bytes, void *stream);
paep_status paep_probe_mfma(int32_t workgroups, int32_t iters, void *sink_dev, size_t sink_bytes, void *stream,
                            double *flops_out);

const char *paep_status_string(paep_status s);

/* Library version as major*10000 + minor*100 + patch. */
int paep_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PAEP_H */

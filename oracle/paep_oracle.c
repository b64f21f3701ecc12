/*
 * CPU oracle for the pre-attention expert predictor.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition that the GPU library is checked
 * against.  Only the tests, the smoke check and the benchmark's CPU-baseline
 * leg may call it; the product never does.  It shares no code, header, table
 * or helper with the HIP implementation.
 *
 * What it computes (paper section 4.1, eq. 3-4, and section 4.3):
 *   the predictor f(X; theta) is two linear layers, d -> r -> E, applied to
 *   the hidden state X that enters a layer's attention block; its output
 *   s in R^E ranks the experts and TopK(s, k) is the prediction.  Section 4.3
 *   places an element-wise function between the two layers (SiLU, or
 *   BatchNorm+GELU whose inference form is an affine map folded into W1, b1
 *   followed by GELU); the abstract and section 1 describe the plain
 *   two-linear form, which is the default here (act = 0).
 *   Softmax is the one of eq. 1; it is monotone, so TopK(softmax(s)) equals
 *   TopK(s) (the ranking-preservation observation of sections 1 and 3.1), and
 *   the selection is made on the raw scores.
 *
 * Arithmetic: every sum is accumulated in double, in ascending index order,
 * with no blocking and no reassociation (compile WITHOUT -ffast-math).
 * Inputs arrive as float arrays that hold the storage values exactly (bf16
 * values widened to float, or fp32).
 *
 * Readings where the paper is silent:
 *   - ties between equal scores go to the lower expert id; the k selected
 *     experts are reported in descending score order;
 *   - probs are softmax over all E scores (max-subtracted), gathered at the
 *     selected experts, not renormalised over the k;
 *   - a NaN score orders as minus infinity;
 *   - round_h = 1 rounds the hidden vector h to bf16 (nearest-even) before
 *     the second layer, modelling a bf16 network in which the first layer's
 *     output is stored as bf16; round_h = 0 keeps h in double.
 *
 * Grouping and scoring have no passage in the paper beyond "select the top-k
 * experts ... for prefetching" (section 4.2, stage three) and the three
 * accuracies of section 5.1; they are written out as their plain definitions:
 * a bincount, an exclusive prefix sum, a stable counting sort, and per-row set
 * comparisons.
 *
 * Pins (tests/test_oracle_pins.py): brute-force selection on tiny inputs,
 * NumPy float64 matmul / argsort / bincount / cumsum, the collapsed form
 * (W2 W1) x, ranking preservation, identity-weight and zero-input special
 * cases, duplicated-row exact ties, and hand-built accuracy cases.
 * The paper prints no worked numeric example of the predictor, so agreement
 * with the paper's own numbers (Table 4) is unpinned: those need its trained
 * weights and collected activations.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_ACT_NONE = 0, ORACLE_ACT_SILU = 1, ORACLE_ACT_GELU = 2 };

/* Nearest-even rounding of a double to the bf16 grid (8 significant bits,
 * exponent range of binary32), returned as double.  One rounding, straight
 * from the double: v = m * 2^e with 0.5 <= |m| < 1, keep 8 bits of m. */
static double round_bf16(double v)
{
    if (v == 0.0 || isnan(v) || isinf(v)) return v;
    int e;
    (void)frexp(v, &e);
    int q = e - 8;                 /* exponent of the last kept bit */
    if (q < -133) q = -133;        /* bf16 subnormal spacing */
    double out = ldexp(nearbyint(ldexp(v, -q)), q);   /* nearbyint: ties to even */
    if (fabs(out) > 3.3895313892515355e38) out = copysign(INFINITY, v);
    return out;
}

double paep_oracle_round_bf16(double v) { return round_bf16(v); }

static double activation(double v, int act)
{
    switch (act) {
    case ORACLE_ACT_SILU: return v / (1.0 + exp(-v));
    case ORACLE_ACT_GELU: return 0.5 * v * (1.0 + erf(v * 0.70710678118654752440));
    default: return v;
    }
}

typedef struct { double z; int32_t e; } scored;

/* total order: higher score first, NaN last, equal scores by lower id */
static int cmp_scored(const void *pa, const void *pb)
{
    const scored *a = (const scored *)pa, *b = (const scored *)pb;
    int an = isnan(a->z), bn = isnan(b->z);
    if (an != bn) return an ? 1 : -1;
    if (!an) {
        if (a->z > b->z) return -1;
        if (a->z < b->z) return 1;
    }
    return (a->e > b->e) - (a->e < b->e);
}

int paep_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * One layer's predictor on T tokens.
 *   x[T,d], W1[r,d], W2[E,r] row-major; b1[r], b2[E] nullable.
 *   idx[T,k] int32, probs[T,k] float, logits[T,E] double (nullable).
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int paep_oracle_predict(int T, int d, int r, int E, int k, int act, int round_h,
                        const float *x, const float *W1, const float *W2,
                        const float *b1, const float *b2,
                        int32_t *idx, float *probs, double *logits)
{
    if (T < 0 || d < 1 || r < 1 || E < 1 || k < 1 || k > E) return -1;
    if (!x || !W1 || !W2 || !idx || !probs) return -1;
    int failed = 0;
#pragma omp parallel
    {
        double *h = (double *)malloc(sizeof(double) * (size_t)r);
        double *z = (double *)malloc(sizeof(double) * (size_t)E);
        scored *s = (scored *)malloc(sizeof(scored) * (size_t)E);
        if (!h || !z || !s) {
#pragma omp atomic write
            failed = 1;
        } else {
#pragma omp for schedule(static)
            for (int t = 0; t < T; ++t) {
                const float *xt = x + (size_t)t * d;
                /* first linear layer */
                for (int j = 0; j < r; ++j) {
                    const float *w = W1 + (size_t)j * d;
                    double acc = 0.0;
                    for (int i = 0; i < d; ++i) acc += (double)w[i] * (double)xt[i];
                    if (b1) acc += (double)b1[j];
                    if (round_h) acc = round_bf16(acc);
                    h[j] = activation(acc, act);
                    if (round_h && act != ORACLE_ACT_NONE) h[j] = round_bf16(h[j]);
                }
                /* second linear layer: the scores s of eq. 3 */
                for (int e = 0; e < E; ++e) {
                    const float *w = W2 + (size_t)e * r;
                    double acc = 0.0;
                    for (int j = 0; j < r; ++j) acc += (double)w[j] * h[j];
                    if (b2) acc += (double)b2[e];
                    z[e] = acc;
                    if (logits) logits[(size_t)t * E + e] = acc;
                }
                /* TopK of eq. 4: full sort of all E scores */
                for (int e = 0; e < E; ++e) { s[e].z = z[e]; s[e].e = e; }
                qsort(s, (size_t)E, sizeof(scored), cmp_scored);
                /* softmax of eq. 1 over all E, gathered at the selection */
                double m = -INFINITY;
                for (int e = 0; e < E; ++e) if (!isnan(z[e]) && z[e] > m) m = z[e];
                double sum = 0.0;
                for (int e = 0; e < E; ++e) if (!isnan(z[e])) sum += exp(z[e] - m);
                for (int j = 0; j < k; ++j) {
                    idx[(size_t)t * k + j] = s[j].e;
                    probs[(size_t)t * k + j] = (float)(exp(s[j].z - m) / sum);
                }
            }
        }
        free(h); free(z); free(s);
    }
    return failed ? -1 : 0;
}

/*
 * Per-expert token grouping of one layer's selections idx[n] (n = T*k flat
 * positions p = t*k + j).
 *   counts[E]     occurrences of each expert id
 *   offsets[E+1]  exclusive prefix sum of counts; offsets[E] = valid entries
 *   token_pos[n]  positions grouped by expert, ascending p inside a group;
 *                 entries past offsets[E] are set to -1
 *   active[E]     ids with counts > 0, ascending; entries past n_active = -1
 *   n_invalid     entries whose id is outside [0, E): skipped everywhere else
 */
int paep_oracle_group(const int32_t *idx, int n, int E,
                      int32_t *counts, int32_t *offsets, int32_t *token_pos,
                      int32_t *active, int32_t *n_active, int32_t *n_invalid)
{
    if (n < 0 || E < 1 || !counts || !offsets || !token_pos || !active || !n_active || !n_invalid)
        return -1;
    if (n > 0 && !idx) return -1;
    for (int e = 0; e < E; ++e) counts[e] = 0;
    int bad = 0;
    for (int p = 0; p < n; ++p) {
        int32_t e = idx[p];
        if (e < 0 || e >= E) ++bad; else ++counts[e];
    }
    offsets[0] = 0;
    for (int e = 0; e < E; ++e) offsets[e + 1] = offsets[e] + counts[e];
    int32_t *cursor = (int32_t *)malloc(sizeof(int32_t) * (size_t)E);
    if (!cursor) return -1;
    for (int e = 0; e < E; ++e) cursor[e] = offsets[e];
    for (int p = 0; p < n; ++p) token_pos[p] = -1;
    for (int p = 0; p < n; ++p) {
        int32_t e = idx[p];
        if (e < 0 || e >= E) continue;
        token_pos[cursor[e]++] = p;
    }
    free(cursor);
    int na = 0;
    for (int e = 0; e < E; ++e) active[e] = -1;
    for (int e = 0; e < E; ++e) if (counts[e] > 0) active[na++] = e;
    *n_active = na;
    *n_invalid = bad;
    return 0;
}

/*
 * Accuracy counters over T rows (paper section 5.1; section 4.1 last
 * paragraph).  Per row, with P = set(idx[t, :k_pred]) and
 * R = set(ref[t, :k_ref]):
 *   counters[0] n_exact  += (P == R)        exact match
 *   counters[1] n_hit    += |P & R|         correctly predicted experts
 *   counters[2] n_cover  += (R subset of P) over-provisioning hit
 *   counters[3] n_top1   += (idx[t,0] in R) top-1
 * A row holding an id outside [0, E) in either array adds nothing.
 * With k_row (may be NULL) row t uses only its first clamp(k_row[t], 1, k_pred)
 * predicted ids: the per-row widths of confidence-driven over-provisioning
 * (section 6, future work: confident rows in exact-match mode, the others
 * over-provisioned).  Ids past that width are not looked at.
 */
int paep_oracle_score(const int32_t *idx, int k_pred, const int32_t *ref, int k_ref,
                      int T, int E, const int32_t *k_row, long long *counters)
{
    if (T < 0 || E < 1 || k_pred < 1 || k_ref < 1 || !counters) return -1;
    if (T > 0 && (!idx || !ref)) return -1;
    unsigned char *inP = (unsigned char *)malloc((size_t)E);
    unsigned char *inR = (unsigned char *)malloc((size_t)E);
    if (!inP || !inR) { free(inP); free(inR); return -1; }
    long long n_exact = 0, n_hit = 0, n_cover = 0, n_top1 = 0;
    for (int t = 0; t < T; ++t) {
        const int32_t *p = idx + (size_t)t * k_pred;
        const int32_t *q = ref + (size_t)t * k_ref;
        int kp = k_pred;
        if (k_row) { kp = k_row[t]; if (kp < 1) kp = 1; if (kp > k_pred) kp = k_pred; }
        int ok = 1;
        for (int j = 0; j < kp; ++j) if (p[j] < 0 || p[j] >= E) ok = 0;
        for (int j = 0; j < k_ref; ++j) if (q[j] < 0 || q[j] >= E) ok = 0;
        if (!ok) continue;
        memset(inP, 0, (size_t)E);
        memset(inR, 0, (size_t)E);
        for (int j = 0; j < kp; ++j) inP[p[j]] = 1;
        for (int j = 0; j < k_ref; ++j) inR[q[j]] = 1;
        int nP = 0, nR = 0, both = 0;
        for (int e = 0; e < E; ++e) { nP += inP[e]; nR += inR[e]; both += (inP[e] & inR[e]); }
        n_hit += both;
        if (both == nR) ++n_cover;
        if (both == nR && both == nP) ++n_exact;
        if (inR[p[0]]) ++n_top1;
    }
    free(inP); free(inR);
    counters[0] = n_exact; counters[1] = n_hit; counters[2] = n_cover; counters[3] = n_top1;
    return 0;
}

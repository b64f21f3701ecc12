// Device-side building blocks shared by the predict kernels (gfx950, wave64).
//
//  * bf16 <-> fp32 conversions on raw bit patterns,
//  * order-preserving packing of (score, expert id) into one 64-bit key, so
//    that an unsigned compare implements "higher score first, equal scores by
//    lower expert id" (the tie rule of the C header),
//  * a sorted top-K list kept in registers, filled by streaming over a row of
//    scores and merged across the lanes that share a row with wave shuffles,
//  * the softmax (eq. 1 of the paper) gathered at the selected experts, or one
//    of the other two confidence scores (softmax over the selected experts
//    only; sigmoid, the function the predictor is trained through, section 4.4),
//  * optionally, the margin between the last selected score and the best one
//    left out (the confidence signal of the paper's closing section),
//  * optionally, one integer atomic per selection into activation counters
//    (the histogram that grouping would compute, fused into the epilogue); the
//    counters may live in LDS (one flush per workgroup) or in global memory.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace paep {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even, by the hardware conversion (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    return __builtin_bit_cast(uint16_t, (__bf16)f);
}

__device__ __forceinline__ float round_to_bf16(float f) { return bf16_bits_to_f32(f32_to_bf16_bits(f)); }

// two floats -> packed pair of bf16 (lo in bits 0..15)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}

__device__ __forceinline__ float apply_act(float v, int act)
{
    if (act == 1) return v / (1.0f + __expf(-v));                        // SiLU
    if (act == 2) return 0.5f * v * (1.0f + erff(v * 0.70710678118654752f));  // exact GELU
    return v;
}

// ---------------------------------------------------------------------------
// (score, expert) -> 64-bit key.  Larger key = better candidate.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t orderable(float f)
{
    f += 0.0f;                                   // -0 -> +0 so the two zeros tie
    uint32_t u = __float_as_uint(f);
    if (f != f) return 0u;                       // NaN orders below -inf
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float unorderable(uint32_t o)
{
    uint32_t u = (o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o;
    return __uint_as_float(u);
}

__device__ __forceinline__ uint64_t make_key(float score, int e)
{
    return ((uint64_t)orderable(score) << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)e);
}
__device__ __forceinline__ int key_expert(uint64_t key) { return (int)(0xFFFFFFFFu - (uint32_t)key); }
__device__ __forceinline__ float key_score(uint64_t key) { return unorderable((uint32_t)(key >> 32)); }

// Sorted (descending) list of the KMAX best keys seen; 0 marks an empty slot
// (every real key is > 0 because its low word is >= 0xFFFFFFFF - PAEP_MAX_E).
template <int KMAX>
struct TopList {
    uint64_t key[KMAX];

    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int j = 0; j < KMAX; ++j) key[j] = 0;
    }
    __device__ __forceinline__ void insert(uint64_t c)
    {
#pragma unroll
        for (int j = 0; j < KMAX; ++j) {
            const bool gt = c > key[j];
            const uint64_t hi = gt ? c : key[j];
            c = gt ? key[j] : c;
            key[j] = hi;
        }
    }
};

// What the epilogue writes besides idx.
//   prob_mode 0: probs[j] = softmax over all E scores, gathered at the selection (eq. 1)
//             1: probs[j] = softmax over the k selected scores only
//             2: probs[j] = sigmoid of the selected score
//   margin:   nullable; margin[row] = score of the last selected expert minus the best
//             score left out (+inf when k = E)
//   counts:   nullable; counts[e] += 1 per selection of expert e (LDS or global)
struct EpilogueOut {
    int prob_mode;
    float* margin_row;
    int32_t* counts_row;
};

__device__ __forceinline__ float sigmoidf_(float v) { return 1.0f / (1.0f + __expf(-v)); }

// Softmax + top-k of one row of E scores held in LDS, computed by G
// consecutive lanes (G a power of two, the group aligned to G).  Lane g of
// the group scans e = g, g+G, ...; the per-lane lists are merged with
// xor-shuffles so that every lane ends with the row's list; lane g writes
// outputs j = g, g+G, ... < k.  KMAX >= k, and >= k + 1 when the margin is
// wanted and k < E.
template <int KMAX, int G>
__device__ __forceinline__ void row_softmax_topk(const float* zrow, int E, int k, int g,
                                                 int32_t* idx_row, float* probs_row, const EpilogueOut& o)
{
    TopList<KMAX> top;
    top.clear();
    for (int e = g; e < E; e += G) top.insert(make_key(zrow[e], e));
#pragma unroll
    for (int mask = 1; mask < G; mask <<= 1) {
        uint64_t other[KMAX];
#pragma unroll
        for (int j = 0; j < KMAX; ++j) other[j] = __shfl_xor((unsigned long long)top.key[j], mask, 64);
#pragma unroll
        for (int j = 0; j < KMAX; ++j) top.insert(other[j]);
    }
    const float m = key_score(top.key[0]);       // row maximum (NaNs order last)
    float s = 0.0f;
    if (o.prob_mode == 0) {
        for (int e = g; e < E; e += G) {
            const float v = zrow[e];
            if (v == v) s += __expf(v - m);
        }
#pragma unroll
        for (int mask = 1; mask < G; mask <<= 1) s += __shfl_xor(s, mask, 64);
    } else if (o.prob_mode == 1) {
#pragma unroll
        for (int j = 0; j < KMAX; ++j)           // every lane holds the whole list: same sum, same order
            if (j < k) s += __expf(key_score(top.key[j]) - m);
    }
    const float inv = 1.0f / s;
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
        if (j < k && (j % G) == g) {
            const float sc = key_score(top.key[j]);
            idx_row[j] = key_expert(top.key[j]);
            probs_row[j] = (o.prob_mode == 2) ? sigmoidf_(sc) : __expf(sc - m) * inv;
            if (o.counts_row) atomicAdd(&o.counts_row[key_expert(top.key[j])], 1);   // activation counts (exact: integers)
        }
    }
    if (o.margin_row && g == 0) {
        float mg = __builtin_inff();
#pragma unroll
        for (int j = 1; j < KMAX; ++j)
            if (j == k && k < E) mg = key_score(top.key[j - 1]) - key_score(top.key[j]);
        *o.margin_row = mg;
    }
}

// Dispatch on the smallest list length that holds k (and the runner-up, when the margin is wanted).
template <int G>
__device__ __forceinline__ void row_softmax_topk_any(const float* zrow, int E, int k, int g,
                                                     int32_t* idx_row, float* probs_row, const EpilogueOut& o)
{
    const int need = k + ((o.margin_row && k < E) ? 1 : 0);
    if (need <= 2)       row_softmax_topk<2, G>(zrow, E, k, g, idx_row, probs_row, o);
    else if (need <= 8)  row_softmax_topk<8, G>(zrow, E, k, g, idx_row, probs_row, o);
    else if (need <= 16) row_softmax_topk<16, G>(zrow, E, k, g, idx_row, probs_row, o);
    else                 row_softmax_topk<33, G>(zrow, E, k, g, idx_row, probs_row, o);
}

// Softmax + top-k of one row held in registers by a whole wave: lane l owns
// z[v] = score of expert l + 64*v (v < NV).  k rounds (one more when the margin
// is wanted) of "wave-wide maximum of the keys still in play"; the lane that
// owns the winner retires it.  Lane j keeps the j-th winner and writes output
// j.  All reductions are xor butterflies, so the result does not depend on
// scheduling.
template <int NV>
__device__ __forceinline__ void wave_softmax_topk(const float (&z)[NV], int E, int k, int lane,
                                                  int32_t* idx_row, float* probs_row, const EpilogueOut& o)
{
    uint64_t key[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int e = lane + 64 * v;
        key[v] = (e < E) ? make_key(z[v], e) : 0ull;
    }
    uint64_t mine = 0ull;
    const int rounds = k + ((o.margin_row && k < E) ? 1 : 0);
    for (int j = 0; j < rounds; ++j) {
        uint64_t best = key[0];
#pragma unroll
        for (int v = 1; v < NV; ++v) best = key[v] > best ? key[v] : best;
#pragma unroll
        for (int mask = 1; mask < 64; mask <<= 1) {
            const uint64_t ot = __shfl_xor((unsigned long long)best, mask, 64);
            best = ot > best ? ot : best;
        }
#pragma unroll
        for (int v = 0; v < NV; ++v) key[v] = (key[v] == best) ? 0ull : key[v];
        if (lane == j) mine = best;
    }
    const float m = key_score(__shfl((unsigned long long)mine, 0, 64));     // row maximum
    const float sc = key_score(mine);
    float s = 0.0f;
    if (o.prob_mode == 0) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int e = lane + 64 * v;
            if (e < E && z[v] == z[v]) s += __expf(z[v] - m);
        }
    } else if (o.prob_mode == 1) {
        if (lane < k) s = __expf(sc - m);
    }
    if (o.prob_mode != 2) {
#pragma unroll
        for (int mask = 1; mask < 64; mask <<= 1) s += __shfl_xor(s, mask, 64);
    }
    if (o.margin_row) {
        const float last = key_score(__shfl((unsigned long long)mine, k - 1, 64));
        const float next = key_score(__shfl((unsigned long long)mine, k < 64 ? k : 63, 64));
        if (lane == 0) *o.margin_row = (k < E) ? last - next : __builtin_inff();
    }
    if (lane < k) {
        idx_row[lane] = key_expert(mine);
        probs_row[lane] = (o.prob_mode == 2) ? sigmoidf_(sc) : __expf(sc - m) / s;
        if (o.counts_row) atomicAdd(&o.counts_row[key_expert(mine)], 1);
    }
}

// The same outputs for a row of at most 128 scores (NV <= 2 per lane), by rank counting:
// every lane learns how many of the row's keys beat its own by walking the 64 lanes' keys
// through scalar registers (v_readlane: no LDS round trip, no dependent chain of shuffles).
// Keys are distinct (the expert id is part of the key), so the ranks are a permutation and the
// lane whose key has rank j < k writes output j.  Selection and order are exactly those of
// wave_softmax_topk; the softmax normaliser is the same butterfly sum.
template <int NV>
__device__ __forceinline__ void wave_softmax_topk_rank(const float (&z)[NV], int E, int k, int lane,
                                                       int32_t* idx_row, float* probs_row, const EpilogueOut& o)
{
    static_assert(NV <= 2, "rank counting is for short rows");
    uint32_t khi[NV], klo[NV];
    int rank[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int e = lane + 64 * v;
        const uint64_t key = (e < E) ? make_key(z[v], e) : 0ull;
        khi[v] = (uint32_t)(key >> 32);
        klo[v] = (uint32_t)key;
        rank[v] = 0;
    }
    for (int j = 0; j < 64; ++j) {                             // uniform: lane j's keys, broadcast
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const uint32_t ohi = (uint32_t)__builtin_amdgcn_readlane((int)khi[u], j);
            const uint32_t olo = (uint32_t)__builtin_amdgcn_readlane((int)klo[u], j);
#pragma unroll
            for (int v = 0; v < NV; ++v) rank[v] += (ohi > khi[v] || (ohi == khi[v] && olo > klo[v])) ? 1 : 0;
        }
    }
    // score of the key with a given rank, for every lane (rank < number of valid keys)
    auto score_of_rank = [&](int want) {
        float found = 0.0f;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const unsigned long long who = __ballot(rank[v] == want && lane + 64 * v < E);
            if (who) found = __uint_as_float((uint32_t)__builtin_amdgcn_readlane(
                         (int)__float_as_uint(z[v]), (int)__builtin_ctzll(who)));
        }
        return found + 0.0f;
    };
    // row maximum as the other routine takes it: the score of the best key (NaNs order last, -0 reads as +0)
    const float m = key_score(((uint64_t)orderable(score_of_rank(0)) << 32));
    float s = 0.0f;
    if (o.prob_mode == 0) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int e = lane + 64 * v;
            if (e < E && z[v] == z[v]) s += __expf(z[v] - m);
        }
    } else if (o.prob_mode == 1) {
#pragma unroll
        for (int v = 0; v < NV; ++v)
            if (lane + 64 * v < E && rank[v] < k) s += __expf(key_score(((uint64_t)khi[v] << 32)) - m);
    }
    if (o.prob_mode != 2) {
#pragma unroll
        for (int mask = 1; mask < 64; mask <<= 1) s += __shfl_xor(s, mask, 64);
    }
    if (o.margin_row) {
        float mg = __builtin_inff();
        if (k < E) mg = key_score(((uint64_t)orderable(score_of_rank(k - 1)) << 32)) -
                        key_score(((uint64_t)orderable(score_of_rank(k)) << 32));
        if (lane == 0) *o.margin_row = mg;
    }
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int e = lane + 64 * v;
        if (e < E && rank[v] < k) {
            const float sc = key_score(((uint64_t)khi[v] << 32));
            idx_row[rank[v]] = e;
            probs_row[rank[v]] = (o.prob_mode == 2) ? sigmoidf_(sc) : __expf(sc - m) / s;
            if (o.counts_row) atomicAdd(&o.counts_row[e], 1);
        }
    }
}

// Same, for kernels that only accept lists of up to 16 (keeps their register budget small):
// k <= 16, and k <= 15 when the margin is wanted and k < E.
template <int G>
__device__ __forceinline__ void row_softmax_topk_upto16(const float* zrow, int E, int k, int g,
                                                        int32_t* idx_row, float* probs_row, const EpilogueOut& o)
{
    const int need = k + ((o.margin_row && k < E) ? 1 : 0);
    if (need <= 2)      row_softmax_topk<2, G>(zrow, E, k, g, idx_row, probs_row, o);
    else if (need <= 8) row_softmax_topk<8, G>(zrow, E, k, g, idx_row, probs_row, o);
    else                row_softmax_topk<16, G>(zrow, E, k, g, idx_row, probs_row, o);
}

}  // namespace paep

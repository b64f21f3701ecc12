// Prefill-shaped predictor (many tokens per layer), bf16 storage: the two
// linear layers of the predictor (paper section 4.3, eq. 3) fused into one
// matrix-core kernel, with softmax and top-k (eq. 1, eq. 4) finished on chip.
//
// A workgroup (4 waves) owns BM = 128 tokens of one layer and walks the inner
// width r in chunks of BN = 128 hidden units.  For a chunk it forms
//     h^T[chunk, tokens] = W1[chunk, :] . x[tokens, :]^T
// with v_mfma_f32_32x32x16_bf16, W1 rows as the A operand and token rows as
// the B operand, both staged through double-buffered, padded LDS tiles of
// BK = 64 along d.  The waves form a 2 x 2 grid over (hidden units, tokens),
// 64 x 64 each.  Written this way round, the accumulator of a 32 x 32 block
// holds, per lane, 16 hidden units of ONE token -- which is exactly what the B
// operand of the next product needs -- so the chunk of h goes, after rounding
// to bf16, bias and activation, straight from the accumulator registers into
//     z^T[E, tokens] += W2[:, chunk] . h^T[chunk, tokens]
// without touching LDS; only the W2 fragments are fetched (two 8-byte loads
// per lane, matching the accumulator's row order).  h and z never reach HBM.
// After the last chunk the two waves that share a token range add their
// partial scores through LDS in a fixed order, and two lanes per token run
// the softmax/top-k epilogue.
#include "paep_device.h"
#include "paep_internal.h"

namespace paep {

static constexpr int PF_THREADS = 256;
static constexpr int BM = 128;          // tokens per workgroup
static constexpr int BN = 128;          // hidden units per chunk
static constexpr int BK = 64;           // d-elements per LDS tile
static constexpr int LDT = BK + 8;      // padded LDS row, bf16 elements
static constexpr int STAGE_ELEMS = (BN + BM) * LDT;
static constexpr int TILE_BYTES = 2 * STAGE_ELEMS * 2;

// EB32: 32-expert blocks (E <= 32 * EB32).  WR: waves along the hidden-unit
// axis of a chunk (2: a 2 x 2 wave grid of 64 x 64 tiles; 1: four waves side by
// side along tokens, 128 x 32 each, which halves the score accumulators per
// wave and is what E = 256 needs to stay in registers).  OCC: workgroups per CU
// the register budget is sized for.
template <int EB32, int WR, int OCC>
__global__ __launch_bounds__(PF_THREADS, OCC) void prefill_kernel(
    int T, int d, int r, int E, int k, int act, int tiles_per_layer, int total_wgs,
    long long xs_, long long w1s, long long w2s,
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ W1, const uint16_t* __restrict__ W2,
    const uint16_t* __restrict__ b1, const uint16_t* __restrict__ b2,
    int32_t* __restrict__ idx, float* __restrict__ probs, float* __restrict__ logits)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    uint16_t* tiles = (uint16_t*)smem_raw;
    float* zs = (float*)smem_raw;                         // reused after the main loop

    // Workgroups are dealt round-robin to the 8 XCDs; remap so that each XCD
    // works through a contiguous range of (layer, token tile) and its L2
    // sees one layer's W1 at a time.
    int wg = blockIdx.x;
    {
        const int per = total_wgs / 8, rem = total_wgs % 8;
        const int xcd = wg % 8, slot = wg / 8;
        wg = xcd * per + (xcd < rem ? xcd : rem) + slot;
    }
    const int layer = wg / tiles_per_layer;
    const int t0 = (wg - layer * tiles_per_layer) * BM;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int WT = 4 / WR;                 // waves along tokens
    constexpr int MI = BN / WR / 32;           // 32-unit blocks per wave
    constexpr int NI = BM / WT / 32;           // 32-token blocks per wave
    constexpr int WM = BN / WR, WN = BM / WT;  // wave tile
    const int wr = wave / WT, wt = wave % WT;
    const int l32 = lane & 31, g = lane >> 5;
    const uint16_t* xl = x + (long long)layer * xs_;
    const uint16_t* W1l = W1 + (long long)layer * w1s;
    const uint16_t* W2l = W2 + (long long)layer * w2s;

    // global -> LDS copy assignment: 4 rows-of-16B per thread and operand
    const int crow = tid >> 3, ccol = (tid & 7) * 8;      // rows crow + 32*q
    const uint16_t* asrc[4];
    const uint16_t* bsrc[4];
    bool bok[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int row = crow + 32 * q;
        asrc[q] = W1l + (long long)row * d + ccol;
        const int tok = t0 + row;
        bok[q] = tok < T;
        bsrc[q] = xl + (long long)(bok[q] ? tok : 0) * d + ccol;
    }

    f32x16 acc1[MI][NI];
    f32x16 acc2[EB32][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc1[mi][ni][i] = 0.f;
#pragma unroll
    for (int eb = 0; eb < EB32; ++eb)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc2[eb][ni][i] = 0.f;

    const int NK = d / BK, NC = r / BN, NT = NK * NC;
    u32x4 ra[4], rb[4];

    auto load_tile = [&](int it) {
        const int kt = it % NK, n = it / NK;
        const long long aoff = (long long)n * BN * d + kt * BK;
        const int boff = kt * BK;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            ra[q] = *(const u32x4*)(asrc[q] + aoff);
            rb[q] = bok[q] ? *(const u32x4*)(bsrc[q] + boff) : u32x4{0u, 0u, 0u, 0u};
        }
    };
    auto store_tile = [&](int stage) {
        uint16_t* As = tiles + stage * STAGE_ELEMS;
        uint16_t* Bs = As + BN * LDT;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            *(u32x4*)(As + (crow + 32 * q) * LDT + ccol) = ra[q];
            *(u32x4*)(Bs + (crow + 32 * q) * LDT + ccol) = rb[q];
        }
    };

    load_tile(0);
    store_tile(0);
    __syncthreads();

    for (int it = 0; it < NT; ++it) {
        const int kt = it % NK, n = it / NK;
        if (it + 1 < NT) load_tile(it + 1);
        {
            const uint16_t* As = tiles + (it & 1) * STAGE_ELEMS + (wr * WM + l32) * LDT + g * 8;
            const uint16_t* Bs = tiles + (it & 1) * STAGE_ELEMS + BN * LDT + (wt * WN + l32) * LDT + g * 8;
#pragma unroll
            for (int ks = 0; ks < BK / 16; ++ks) {
                bf16x8 a[MI], b[NI];
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
                    a[mi] = __builtin_bit_cast(bf16x8, *(const u32x4*)(As + mi * 32 * LDT + ks * 16));
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    b[ni] = __builtin_bit_cast(bf16x8, *(const u32x4*)(Bs + ni * 32 * LDT + ks * 16));
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni)
                        acc1[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mi], b[ni], acc1[mi][ni], 0, 0, 0);
            }
        }
        if (it + 1 < NT) store_tile((it + 1) & 1);
        __syncthreads();

        if (kt == NK - 1) {
            // chunk n of h is complete in acc1: feed it to the second layer.
            // acc1[mi][ni][i] = h[token wt*WN + ni*32 + l32]
            //                    [unit n*BN + wr*WM + mi*32 + 8*(i/4) + 4*g + i%4]
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const int unit0 = n * BN + wr * WM + mi * 32 + 16 * s + 4 * g;   // units unit0+0..3, unit0+8..11
                    float bias[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) bias[i] = 0.f;
                    if (b1) {
#pragma unroll
                        for (int i = 0; i < 8; ++i)
                            bias[i] = bf16_bits_to_f32(b1[(long long)layer * r + unit0 + (i & 3) + 8 * (i >> 2)]);
                    }
                    bf16x8 hb[NI];
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni) {
                        float v[8];
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            float h = round_to_bf16(acc1[mi][ni][8 * s + i] + bias[i]);
                            if (act != 0) h = round_to_bf16(apply_act(h, act));
                            v[i] = h;
                        }
                        u32x4 pk = u32x4{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]),
                                         pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])};
                        hb[ni] = __builtin_bit_cast(bf16x8, pk);
                    }
#pragma unroll
                    for (int eb = 0; eb < EB32; ++eb) {
                        const int e = eb * 32 + l32;
                        u32x4 wv = u32x4{0u, 0u, 0u, 0u};
                        if (e < E) {
                            const uint16_t* wp = W2l + (long long)e * r + unit0;
                            const u32x2 lo = *(const u32x2*)wp;
                            const u32x2 hi = *(const u32x2*)(wp + 8);
                            wv = u32x4{lo[0], lo[1], hi[0], hi[1]};
                        }
                        const bf16x8 wa = __builtin_bit_cast(bf16x8, wv);
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni)
                            acc2[eb][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa, hb[ni], acc2[eb][ni], 0, 0, 0);
                    }
                }
            }
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc1[mi][ni][i] = 0.f;
        }
    }

    // acc2[eb][ni][i] = partial score of token wt*WN + ni*32 + l32,
    //                   expert eb*32 + 8*(i/4) + 4*g + i%4, over this wave's hidden units.
    // Waves that share tokens add their parts through LDS, wr = 0 first.
    const int ZP = E + 1;
#pragma unroll
    for (int pass = 0; pass < WR; ++pass) {
        if (wr == pass) {
#pragma unroll
            for (int eb = 0; eb < EB32; ++eb)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int e = eb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
                        const int tl = wt * WN + ni * 32 + l32;
                        if (e < E) {
                            float v = acc2[eb][ni][i];
                            if (pass == 0) {
                                if (b2) v += bf16_bits_to_f32(b2[(long long)layer * E + e]);
                            } else {
                                v = zs[tl * ZP + e] + v;
                            }
                            zs[tl * ZP + e] = v;
                        }
                    }
        }
        __syncthreads();
    }

    if (logits) {
        for (int i = tid; i < BM * E; i += PF_THREADS) {
            const int tl = i / E, e = i - tl * E;
            if (t0 + tl < T) logits[((long long)layer * T + t0 + tl) * E + e] = zs[tl * ZP + e];
        }
    }
    {
        const int tl = tid >> 1, gg = tid & 1;
        // both lanes of a pair take the same branch (same token)
        if (t0 + tl < T) {
            const long long row = (long long)layer * T + t0 + tl;
            row_softmax_topk_upto16<2>(zs + tl * ZP, E, k, gg, idx + row * k, probs + row * k);
        }
    }
}

static size_t prefill_lds_bytes(int E)
{
    const size_t z = sizeof(float) * (size_t)BM * (size_t)(E + 1);
    return z > (size_t)TILE_BYTES ? z : (size_t)TILE_BYTES;
}

bool prefill_supported(const PredictArgs& a)
{
    return a.dtype == 1 && a.T >= 1 && a.d % BK == 0 && a.r % BN == 0 && a.E <= 256 && a.k <= 16 &&
           prefill_lds_bytes(a.E) <= 160 * 1024;
}

hipError_t launch_predict_prefill(const PredictArgs& a)
{
    const int tiles = (a.T + BM - 1) / BM;
    const int total = tiles * a.L;
    const size_t lds = prefill_lds_bytes(a.E);
    hipError_t err;
#define PAEP_LAUNCH_PF(EBV, WRV, OCCV)                                                               \
    do {                                                                                             \
        auto kern = prefill_kernel<EBV, WRV, OCCV>;                                                           \
        err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,     \
                                  (int)lds);                                                         \
        if (err != hipSuccess) return err;                                                           \
        hipLaunchKernelGGL(kern, dim3(total), dim3(PF_THREADS), lds, a.stream, a.T, a.d, a.r, a.E,   \
                           a.k, a.act, tiles, total, a.x_stride, a.w1_stride, a.w2_stride,           \
                           (const uint16_t*)a.x, (const uint16_t*)a.W1, (const uint16_t*)a.W2,       \
                           (const uint16_t*)a.b1, (const uint16_t*)a.b2, a.idx, a.probs, a.logits);  \
    } while (0)
    if (a.E <= 32)       PAEP_LAUNCH_PF(1, 2, 2);
    else if (a.E <= 64)  PAEP_LAUNCH_PF(2, 2, 2);
    else if (a.E <= 128) PAEP_LAUNCH_PF(4, 2, 1);
    else                 PAEP_LAUNCH_PF(8, 1, 1);
#undef PAEP_LAUNCH_PF
    return hipGetLastError();
}

}  // namespace paep

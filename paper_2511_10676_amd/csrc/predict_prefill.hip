// Prefill-shaped predictor (many tokens per layer), bf16 storage: the two
// linear layers of the predictor (paper section 4.3, eq. 3) fused into one
// matrix-core kernel, with softmax and top-k (eq. 1, eq. 4) finished on chip.
//
// A workgroup owns BM tokens of one layer and walks the inner width r in chunks
// of BN hidden units (tile shapes: PfCfg below).  For a chunk it forms
//     h^T[chunk, tokens] = W1[chunk, :] . x[tokens, :]^T
// with v_mfma_f32_32x32x16_bf16, W1 rows as the A operand and token rows as
// the B operand, both copied global -> LDS without staging registers into a
// ring of XOR-swizzled stages of BK elements along d.  The waves form a
// WR x WT grid over (hidden units, tokens).  Written this way round, the
// accumulator of a 32 x 32 block holds, per lane, 16 hidden units of ONE
// token -- which is exactly what the B operand of the next product needs -- so
// the chunk of h goes, after bias, activation and rounding to bf16, straight
// from the accumulator registers into
//     z^T[E, tokens] += W2[:, chunk] . h^T[chunk, tokens]
// without touching LDS; the W2 fragments come from a copy of the chunk's W2
// slice that was brought into LDS while the chunk's first product ran (two
// 8-byte reads per lane, matching the accumulator's row order).  h and z never
// reach HBM.
// After the last chunk the waves that share a token range add their partial
// scores through LDS in a fixed order, and one to four lanes per token run the
// softmax/top-k epilogue.  r may also be split over several workgroups per
// token tile; their partial score tiles then meet in a workspace and the
// workgroup that finishes last adds them in a fixed order.
#include <type_traits>

#include "paep_device.h"
#include "paep_internal.h"

namespace paep {

// s_waitcnt immediate that waits for vmcnt <= n and nothing else (gfx9 encoding)
#define PAEP_VMCNT(n) ((((n) & 0xF) | (((n) >> 4) << 14)) | 0x0F70)

typedef void __attribute__((address_space(3)))* lptr_t;

template <int V> using IC = std::integral_constant<int, V>;
template <int N, class F> __device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(IC<N - 1>{});
    }
}

// Tile configuration.
//   BM tokens x BN hidden units per workgroup and chunk, BK elements of d per
//   LDS tile, NS LDS stages; WR x WT waves over (hidden units, tokens); OCC
//   workgroups per CU the register budget is sized for.
// Tiles travel global -> LDS with buffer_load_dwordx4 ... lds (no staging
// registers), NS stages deep, so a tile is requested two or three iterations
// before it is used.  An LDS tile row holds BK bf16 = CPR chunks of 16 bytes; chunk c of
// row R sits in slot c ^ swz(R), chosen so that the 16-lane groups of a
// ds_read_b128 touch 64 distinct banks.  The swizzle is applied on the global
// side of the copy (a lane picks which chunk it fetches), because the LDS side
// of that instruction is fixed to lane * 16 bytes from a wave-uniform base.
//   W2L: the chunk's slice of W2 (all experts x BN hidden units) is copied to LDS
//   a chunk ahead, behind the stages, and the second layer reads its fragments
//   from there.  Read straight from global memory, every fragment of the second
//   layer is a load the next matrix instruction waits for (no registers are
//   free to request them ahead): measured, the second layer then takes 16% of
//   the loop with 64 experts and 36-39% with 128 and 256.
template <int BM_, int BN_, int BK_, int NS_, int WR_, int WT_, int OCC_, bool W2L_ = true>
struct PfCfg {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, NS = NS_, WR = WR_, WT = WT_, OCC = OCC_;
    static constexpr bool W2L = W2L_;
    static constexpr int CW = BN / 8;                       // 16-byte chunks per row of the W2 slice
    static constexpr int RPIW = 64 / CW;                    // slice rows moved by one copy instruction
    static constexpr int NW = WR * WT, THREADS = 64 * NW;
    static constexpr int WM = BN / WR, WN = BM / WT;        // wave tile: hidden units x tokens
    static constexpr int MI = WM / 32, NI = WN / 32;        // 32 x 32 blocks per wave
    static constexpr int CPR = BK / 8;                      // 16-byte chunks per tile row
    static constexpr int RPI = 64 / CPR;                    // tile rows moved by one copy instruction
    static constexpr int AJ = BN / RPI / NW, BJ = BM / RPI / NW;   // copy instructions per wave and tile
    static constexpr int STAGE_ELEMS = (BN + BM) * BK;
    static constexpr int TILE_BYTES = NS * STAGE_ELEMS * 2;
    static_assert(BK == 32 || BK == 64, "BK");
    static_assert(AJ >= 1 && BJ >= 1 && AJ * RPI * NW == BN && BJ * RPI * NW == BM, "copy split");
    static_assert(MI >= 1 && NI >= 1, "wave tile");
    static_assert((AJ + BJ) * NS <= 56, "vmcnt budget");
    static __device__ __forceinline__ int swz(int row) { return BK == 32 ? ((row >> 2) & 3) : ((row >> 1) & 7); }
};

// Token rows of the score tile that are staged in LDS at once (<= 128 KB).
template <class C, int EB32>
struct PfZRows {
    static constexpr int value = (C::BM * (EB32 * 32 + 1) * 4 > 128 * 1024) ? C::BM / 2 : C::BM;
};

// EB32: 32-expert blocks (E <= 32 * EB32).
template <class C, int EB32>
__global__ __launch_bounds__(C::THREADS, C::OCC) void prefill_kernel(
    int T, int d, int r, int E, int k, int act, int tiles_per_layer, int main_wgs, int main_groups, int tail_wgs,
    int tail_groups, int split_tile0, int nchunks,
    long long xs_, long long w1s, long long w2s,
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ W1, const uint16_t* __restrict__ W2,
    const uint16_t* __restrict__ b1, const uint16_t* __restrict__ b2,
    int32_t* __restrict__ idx, float* __restrict__ probs, float* __restrict__ logits,
    float* __restrict__ zpart, int* __restrict__ tickets, int32_t* __restrict__ counts,
    int prob_mode, float* __restrict__ margin)
{
    constexpr int BM = C::BM, BN = C::BN, BK = C::BK, NS = C::NS, WR = C::WR, WT = C::WT;
    constexpr int WM = C::WM, WN = C::WN, MI = C::MI, NI = C::NI, CPR = C::CPR, RPI = C::RPI;
    constexpr int AJ = C::AJ, BJ = C::BJ, STAGE_ELEMS = C::STAGE_ELEMS;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    uint16_t* tiles = (uint16_t*)smem_raw;
    float* zs = (float*)smem_raw;                         // reused after the main loop

    // A work item is (layer, token tile, group of r-chunks).  Workgroups are
    // dealt round-robin to the 8 XCDs; remap so that each XCD walks a contiguous
    // range of items with the chunk group varying fastest.  The workgroups that
    // run together on an XCD then cover a few token tiles times all chunk groups
    // of one layer: every x tile is shared by `groups` workgroups and every W1
    // chunk by several token tiles through that XCD's L2, instead of each
    // workgroup pulling its own x tile from far memory once per chunk.
    // The grid has two parts: `main_wgs` workgroups that run the first tiles with `main_groups`
    // workgroups per tile, then `tail_wgs` that run the remaining tiles with `tail_groups` each (the
    // tiles that would otherwise form a last, partly filled round of whole-tile workgroups are cut
    // finer so that every CU stays busy to the end).  Each part is remapped by itself.
    int wg = blockIdx.x;
    const bool in_tail = wg >= main_wgs;
    {
        const int part_wgs = in_tail ? tail_wgs : main_wgs;
        if (in_tail) wg -= main_wgs;
        const int per = part_wgs / 8, rem = part_wgs % 8;
        const int xcd = wg % 8, slot = wg / 8;
        wg = xcd * per + (xcd < rem ? xcd : rem) + slot;
    }
    const int groups = in_tail ? tail_groups : main_groups;
    const int cpg = nchunks / groups;
    const int cg = wg % groups;
    const int tile_id = (in_tail ? main_wgs / main_groups : 0) + wg / groups;   // layer * tiles_per_layer + token tile
    const int layer = tile_id / tiles_per_layer;
    const int t0 = (tile_id - layer * tiles_per_layer) * BM;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
    const int wr = wave / WT, wt = wave % WT;
    const int l32 = lane & 31, g = lane >> 5;
    const uint16_t* xl = x + (long long)layer * xs_;
    const uint16_t* W1l = W1 + (long long)layer * w1s;
    const uint16_t* W2l = W2 + (long long)layer * w2s;

    // global -> LDS copy assignment: per tile, wave w moves rows
    // (w*AJ + j)*RPI .. +RPI of the W1 tile (j < AJ) and likewise of the token
    // tile; lane l supplies row l / CPR, slot l % CPR of its instruction.
    // Addresses are a wave-uniform base plus a 32-bit byte offset per lane.
    uint32_t alane[AJ], blane[BJ];
#pragma unroll
    for (int j = 0; j < AJ; ++j) {
        const int row = (wave * AJ + j) * RPI + lane / CPR;
        const int chunk = (lane % CPR) ^ C::swz(row);
        alane[j] = (uint32_t)(row * d + chunk * 8) * 2u;
    }
#pragma unroll
    for (int j = 0; j < BJ; ++j) {
        const int row = (wave * BJ + j) * RPI + lane / CPR;
        const int chunk = (lane % CPR) ^ C::swz(row);
        blane[j] = (uint32_t)(row * d + chunk * 8) * 2u;   // rows past the end of the layer read as zero
    }
    const char* xtile = (const char*)(xl + (long long)t0 * d);

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

    const int NK = d / BK;
    const int n_begin = cg * cpg, n_end = n_begin + cpg;     // this work item's chunks of r
    // The slice's copies are requested after the first barrier of a chunk and must have landed, for every wave,
    // before a barrier that precedes the chunk's second layer.  A wave's wait before the barrier of tile i lets only
    // the copies of the NS - 1 youngest tiles stay in flight, so with enough tiles per chunk that holds by itself.
    const bool w2_sync = NK < NS + 2;

    // Global -> LDS requests for the next tile in sequence, one copy instruction
    // ("piece") at a time so that they can be spread between the MFMAs instead
    // of holding a wave in a burst of memory instructions.  Pieces 0..AJ-1 move
    // this wave's rows of the W1 tile, AJ..AJ+BJ-1 its rows of the token tile.
    // issue_advance() steps the tile coordinates (counters, no division); past
    // the end it stays on the last tile, which is then re-read into a stage
    // nobody looks at again: the number of copies in flight stays constant, so
    // one s_waitcnt immediate serves every iteration.
    constexpr int NP = AJ + BJ;
    int iss_kt = 0, iss_n = n_begin;
    // Buffer-addressed copies (buffer_load_dwordx4 ... lds): base and bounds in a
    // scalar resource, a 32-bit lane offset, a scalar tile offset.  Token rows
    // past the end of the layer fall outside the resource and read as zero.  (The
    // flat-addressed form of this instruction makes the compiler wait for every
    // outstanding LDS read before the next MFMA, which serialises the pipeline.)
    const __amdgpu_buffer_rsrc_t rsrc_a =
        __builtin_amdgcn_make_buffer_rsrc((void*)W1l, 0, (int)((long long)r * d * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_b =
        __builtin_amdgcn_make_buffer_rsrc((void*)xtile, 0, (int)((long long)(T - t0) * d * 2), 0x00020000);
    auto issue_piece = [&](int slot, auto q_c) {
        constexpr int q = decltype(q_c)::value;
        uint16_t* As = tiles + slot * STAGE_ELEMS;
        if constexpr (q < AJ) {
            const int soff = (iss_n * BN * d + iss_kt * BK) * 2;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, (lptr_t)(As + (wave * AJ + q) * RPI * BK), 16,
                                                     (int)alane[q], soff, 0, 0);
        } else {
            const int soff = iss_kt * BK * 2;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_b, (lptr_t)(As + BN * BK + (wave * BJ + (q - AJ)) * RPI * BK),
                                                     16, (int)blane[q - AJ], soff, 0, 0);
        }
    };
    auto issue_advance = [&]() {
        if (iss_kt + 1 < NK) ++iss_kt;
        else if (iss_n + 1 < n_end) { iss_kt = 0; ++iss_n; }
    };
    auto issue_tile = [&](int slot) {
        static_for<NP>([&](auto q_c) { issue_piece(slot, q_c); });
        issue_advance();
    };

    // The W2 slice of a chunk in LDS, behind the stages: row e (expert) holds BN hidden units = CW
    // chunks of 16 bytes, chunk c in slot c ^ (e % CW) (swizzled on the global side of the copy, like
    // the tiles).  Rows past E lie outside the buffer resource and arrive as zeros.
    constexpr int CW = C::CW, RPIW = C::RPIW, W2ROWS = EB32 * 32;
    constexpr int W2J = C::W2L ? W2ROWS / RPIW / C::NW : 0;     // copy instructions per wave and slice
    static_assert(!C::W2L || W2J * RPIW * C::NW == W2ROWS, "W2 slice copy split");
    uint16_t* w2lds = tiles + NS * STAGE_ELEMS;
    const __amdgpu_buffer_rsrc_t rsrc_w2 =
        __builtin_amdgcn_make_buffer_rsrc((void*)W2l, 0, (int)((long long)E * r * 2), 0x00020000);
    auto issue_w2 = [&](int n) {
        if constexpr (C::W2L) {
#pragma unroll
            for (int j = 0; j < W2J; ++j) {
                const int row0 = (wave * W2J + j) * RPIW;
                const int e = row0 + lane / CW;
                const int chunk = (lane % CW) ^ (e % CW);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_w2, (lptr_t)(w2lds + row0 * BN), 16,
                                                         (int)((uint32_t)(e * r + chunk * 8) * 2u), n * BN * 2, 0, 0);
            }
        }
    };

    // LDS read offsets (elements) of this lane's first A / B fragment at k-step 0.
    // Block mi (ni) is a constant mi*32*BK further on (the swizzle only looks at
    // row bits below 32), and k-step ks flips slot bits: offset ^ (ks * 16).
    constexpr int KS = BK / 16;
    const int arow0 = wr * WM + l32, brow0 = wt * WN + l32;
    const int aoff0 = arow0 * BK + ((g ^ C::swz(arow0)) * 8);
    const int boff0 = BN * BK + brow0 * BK + ((g ^ C::swz(brow0)) * 8);

    // Fragment registers.  B fragments are double-buffered by k-step parity; A
    // fragments are single-buffered and refilled one by one as soon as the
    // MFMAs that use them have been issued ("rolling"), so that LDS reads for
    // the next k-step run under the current k-step's matrix work.
    bf16x8 fa[MI], fb[2][NI];
    auto read_a = [&](const uint16_t* st, auto ks_c, auto mi_c) {
        constexpr int ks = decltype(ks_c)::value, mi = decltype(mi_c)::value;
        fa[mi] = __builtin_bit_cast(bf16x8, *(const u32x4*)(st + ((aoff0 ^ (ks * 16)) + mi * 32 * BK)));
    };
    auto read_b = [&](const uint16_t* st, auto ks_c, auto buf_c) {
        constexpr int ks = decltype(ks_c)::value, buf = decltype(buf_c)::value;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
            fb[buf][ni] = __builtin_bit_cast(bf16x8, *(const u32x4*)(st + ((boff0 ^ (ks * 16)) + ni * 32 * BK)));
    };
    auto mfma_row = [&](auto mi_c, auto buf_c) {
        constexpr int mi = decltype(mi_c)::value, buf = decltype(buf_c)::value;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
            acc1[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mi], fb[buf][ni], acc1[mi][ni], 0, 0, 0);
    };
    auto wg_barrier = [&]() {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    // Chunk n of h is complete in acc1: round it to bf16 and feed it to the
    // second layer straight from the accumulator registers, then clear acc1.
    // acc1[mi][ni][i] = h[token wt*WN + ni*32 + l32]
    //                    [unit n*BN + wr*WM + mi*32 + 8*(i/4) + 4*g + i%4]
    // W2 fragments are requested first (with few enough experts that they fit in
    // registers beside the conversion's temporaries), so that their latency runs
    // under the rounding arithmetic; rows past E are clamped for the address and
    // zeroed by a select, which keeps the loads free of branches.
    constexpr bool EARLY_W2 = !C::W2L && (EB32 <= 4) && (MI * NI + EB32 * NI < 12);    // accumulators leave room for the fragments
    auto w2_fragment = [&](int eb, int unit0) {
        const int e = eb * 32 + l32;
        const uint16_t* wp = W2l + (long long)(e < E ? e : E - 1) * r + unit0;
        const u32x2 lo = *(const u32x2*)wp;
        const u32x2 hi = *(const u32x2*)(wp + 8);
        const bool ok = e < E;
        return u32x4{ok ? lo[0] : 0u, ok ? lo[1] : 0u, ok ? hi[0] : 0u, ok ? hi[1] : 0u};
    };
    // the same fragment out of the LDS copy of the slice; ubase = first hidden unit of the 16-unit step inside the chunk
    auto w2_fragment_lds = [&](int eb, int ubase) {
        const int e = eb * 32 + l32;
        const char* row = (const char*)w2lds + e * (BN * 2) + 8 * g;
        const int c0 = ubase >> 3, sw = e % CW;
        const u32x2 lo = *(const u32x2*)(row + ((c0 ^ sw) << 4));
        const u32x2 hi = *(const u32x2*)(row + (((c0 + 1) ^ sw) << 4));
        return u32x4{lo[0], lo[1], hi[0], hi[1]};
    };
    auto second_layer = [&](int n) {
        const bool plain = (act == 0) && (b1 == nullptr);     // uniform: no bias, identity activation
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int unit0 = n * BN + wr * WM + mi * 32 + 16 * s + 4 * g;   // units unit0+0..3, unit0+8..11
                u32x4 wv[EB32];
                if constexpr (EARLY_W2) {
#pragma unroll
                    for (int eb = 0; eb < EB32; ++eb) wv[eb] = w2_fragment(eb, unit0);
                }
                bf16x8 hb[NI];
                if (plain) {
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni) {
                        const f32x16& a = acc1[mi][ni];
                        u32x4 pk = u32x4{pack_bf16x2(a[8 * s + 0], a[8 * s + 1]), pack_bf16x2(a[8 * s + 2], a[8 * s + 3]),
                                         pack_bf16x2(a[8 * s + 4], a[8 * s + 5]), pack_bf16x2(a[8 * s + 6], a[8 * s + 7])};
                        hb[ni] = __builtin_bit_cast(bf16x8, pk);
                    }
                } else {
                    float bias[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) bias[i] = 0.f;
                    if (b1) {
#pragma unroll
                        for (int i = 0; i < 8; ++i)
                            bias[i] = bf16_bits_to_f32(b1[(long long)layer * r + unit0 + (i & 3) + 8 * (i >> 2)]);
                    }
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni) {
                        float v[8];
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            float h = acc1[mi][ni][8 * s + i] + bias[i];
                            if (act != 0) h = apply_act(round_to_bf16(h), act);   // h is stored as bf16 before the activation
                            v[i] = h;                                            // rounded to bf16 by the packing below
                        }
                        u32x4 pk = u32x4{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]),
                                         pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])};
                        hb[ni] = __builtin_bit_cast(bf16x8, pk);
                    }
                }
                if constexpr (C::W2L) {
                    // fragments from LDS, the next one requested before the current one is multiplied
                    const int ubase = wr * WM + mi * 32 + 16 * s;
                    u32x4 cur = w2_fragment_lds(0, ubase);
#pragma unroll
                    for (int eb = 0; eb < EB32; ++eb) {
                        u32x4 nxt = cur;
                        if (eb + 1 < EB32) nxt = w2_fragment_lds(eb + 1, ubase);
                        const bf16x8 wa = __builtin_bit_cast(bf16x8, cur);
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni)
                            acc2[eb][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa, hb[ni], acc2[eb][ni], 0, 0, 0);
                        cur = nxt;
                    }
                } else {
#pragma unroll
                    for (int eb = 0; eb < EB32; ++eb) {
                        if constexpr (!EARLY_W2) wv[eb] = w2_fragment(eb, unit0);
                        const bf16x8 wa = __builtin_bit_cast(bf16x8, wv[eb]);
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni)
                            acc2[eb][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa, hb[ni], acc2[eb][ni], 0, 0, 0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);          // keep the W2 fetches of later steps from piling up in registers
            }
        }
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc1[mi][ni][i] = 0.f;
    };

    // Stage recycling.  With four or more stages (LAG) the stage refilled after
    // the barrier inside tile `it` is the one tile it-1 used: every wave has
    // certainly finished reading it (its fragments fed MFMAs issued before this
    // barrier), so no wait on outstanding LDS reads is needed at the barrier.
    // With fewer stages the current tile's own stage is refilled, which requires
    // this wave's last fragment reads to have completed first.
    constexpr bool LAG = (NS >= 4);
    constexpr bool LATE_FRAGS = (EB32 >= 8);
    constexpr bool DEFER = (NS >= 3) && (NP % 2 == 0) && (NP / 2 <= MI);
    constexpr int HALF = NP / 2;
    constexpr int PRO = LAG ? NS - 1 : NS;                        // tiles requested before the loop
    constexpr int WAIT_LDS = 0xC07F;                              // lgkmcnt(0) only
    // next tile landed: the younger tiles that may still be in flight
    constexpr int WAIT_NEXT = LAG ? PAEP_VMCNT(NP * (NS - 3)) : (PAEP_VMCNT(NP * (NS - 2)) & WAIT_LDS);

    // PRO tiles requested up front; tile 0 has landed for everyone after the barrier.
    // (With DEFER the coordinates stay on the last requested tile: the main loop's
    // first deferred half-copy repeats that tile's second half, then advances.)
    issue_w2(n_begin);                                            // oldest copies in flight: landed once tile 0 has
#pragma unroll
    for (int p = 0; p < PRO; ++p) {
        static_for<NP>([&](auto q_c) { issue_piece(p, q_c); });
        if (p + 1 < PRO || !DEFER) issue_advance();
    }
    __builtin_amdgcn_s_waitcnt(PAEP_VMCNT(NP * (PRO - 1)));
    wg_barrier();

    // Main loop.  Per k-step: request the next step's B fragments, then for each
    // 32-unit block issue its MFMAs and immediately refill its A fragment for the
    // next step.  On a tile's last k-step the "next step" is the first of the next
    // tile, so the workgroup barrier that hands over LDS stages sits at the top of
    // that step: by then this wave has all its fragments of the current tile in
    // registers and its copies of the next tile have landed.  The copies that
    // refill the stage freed by that barrier are dealt out one per MFMA pair-row:
    // the first half during this last k-step, the second half during the first
    // k-step of the next tile (DEFER), or all at once when there are only two
    // stages and the data is needed one tile later.
    int slot = 0;                                                 // stage of the tile being multiplied
    int free_slot = LAG ? NS - 1 : 0;                             // stage that the next barrier releases for refilling
    int fill_slot = PRO - 1;                                      // stage whose second half of copies is pending
    {
        static_for<MI>([&](auto mi_c) { read_a(tiles, IC<0>{}, mi_c); });
        read_b(tiles, IC<0>{}, IC<0>{});
        __builtin_amdgcn_s_waitcnt(WAIT_LDS);                     // nothing pending on loop entry
    }
    for (int n = n_begin; n < n_end; ++n) {
        for (int kt = 0; kt < NK; ++kt) {
            const uint16_t* st = tiles + slot * STAGE_ELEMS;
            const int nslot = (slot + 1 == NS) ? 0 : slot + 1;
            const uint16_t* stn = tiles + nslot * STAGE_ELEMS;
            static_for<KS>([&](auto ks_c) {
                constexpr int ks = decltype(ks_c)::value;
                constexpr int cur = ks & 1, nxt = cur ^ 1;
                if constexpr (ks + 1 < KS) {
                    read_b(st, IC<ks + 1>{}, IC<nxt>{});
                    __builtin_amdgcn_sched_barrier(0);
                    static_for<MI>([&](auto mi_c) {
                        constexpr int mi = decltype(mi_c)::value;
                        mfma_row(mi_c, IC<cur>{});
                        __builtin_amdgcn_sched_barrier(0);
                        if constexpr (DEFER && ks == 0 && mi < HALF) {
                            // second half of the copies for the stage released one tile ago
                            // (on the very first tile this repeats copies the prologue made: harmless)
                            issue_piece(fill_slot, IC<HALF + mi>{});
                            if constexpr (mi == HALF - 1) issue_advance();
                        }
                        read_a(st, IC<ks + 1>{}, mi_c);
                        __builtin_amdgcn_sched_barrier(0);
                    });
                } else {
                    __builtin_amdgcn_s_waitcnt(WAIT_NEXT);
                    wg_barrier();
                    // Every wave is past the previous chunk's second layer here, so the slice in LDS may
                    // be replaced by this chunk's; it is read at the end of the chunk, NK - 1 tiles later.
                    if (C::W2L && kt == 0 && n > n_begin) issue_w2(n);
                    if constexpr (!DEFER) issue_tile(free_slot);
                    // With many experts the score accumulators leave no room to carry the next
                    // tile's first fragments across the second layer: fetch them after it instead.
                    const bool prefetch = !(LATE_FRAGS && kt == NK - 1);
                    if (prefetch) read_b(stn, IC<0>{}, IC<nxt>{});
                    __builtin_amdgcn_sched_barrier(0);
                    static_for<MI>([&](auto mi_c) {
                        constexpr int mi = decltype(mi_c)::value;
                        mfma_row(mi_c, IC<cur>{});
                        __builtin_amdgcn_sched_barrier(0);
                        if constexpr (DEFER && mi < HALF) issue_piece(free_slot, IC<mi>{});
                        if (prefetch) read_a(stn, IC<0>{}, mi_c);
                        __builtin_amdgcn_sched_barrier(0);
                    });
                    fill_slot = free_slot;
                }
            });
            free_slot = LAG ? slot : nslot;
            slot = nslot;
        }
        if (C::W2L && w2_sync) {
            // few tiles per chunk: the slice's copies may still be among the youngest in flight
            __builtin_amdgcn_s_waitcnt(PAEP_VMCNT(0));
            wg_barrier();
        }
        second_layer(n);
        if constexpr (LATE_FRAGS) {
            const uint16_t* stc = tiles + slot * STAGE_ELEMS;
            static_for<MI>([&](auto mi_c) { read_a(stc, IC<0>{}, mi_c); });
            read_b(stc, IC<0>{}, IC<(((KS - 1) & 1) ^ 1)>{});
        }
        __builtin_amdgcn_s_waitcnt(WAIT_LDS);                     // next tile's first fragments have landed
    }
    __syncthreads();                                       // all tile reads done before LDS is reused

    // Activation counters of this workgroup's rows, kept in LDS behind the score
    // tile and flushed to the layer's counts once at the end: at most E global
    // atomics per workgroup instead of one per selection.
    int32_t* cnt_lds = (int32_t*)(smem_raw + sizeof(float) * (size_t)PfZRows<C, EB32>::value * (size_t)(E + 1));
    if (counts)
        for (int e = tid; e < E; e += C::THREADS) cnt_lds[e] = 0;
    auto flush_counts = [&]() {                              // after a barrier that follows the last row's epilogue
        if (counts)
            for (int e = tid; e < E; e += C::THREADS) {
                const int c = cnt_lds[e];
                if (c) atomicAdd(&counts[(long long)layer * E + e], c);
            }
    };

    // acc2[eb][ni][i] = partial score of token wt*WN + ni*32 + l32,
    //                   expert eb*32 + 8*(i/4) + 4*g + i%4, over this wave's hidden units.
    // The score tile goes to LDS ZROWS tokens at a time (all of it unless E is
    // large); waves that share tokens add their parts there, wr = 0 first.
    constexpr int ZROWS = PfZRows<C, EB32>::value;
    constexpr int ZG = C::THREADS / ZROWS;                 // lanes per token row in the epilogue
    static_assert(ZROWS % WN == 0 && (ZG == 1 || ZG == 2 || ZG == 4), "epilogue split");
    const int ZP = E + 1;
    const bool split = groups > 1;

    // registers -> zs for token rows [zp*ZROWS, (zp+1)*ZROWS); b2 is added here only when r is not split
    auto regs_to_lds = [&](int zp) {
        const bool mine = (wt * WN) / ZROWS == zp;
#pragma unroll
        for (int pass = 0; pass < WR; ++pass) {
            if (mine && wr == pass) {
#pragma unroll
                for (int eb = 0; eb < EB32; ++eb)
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            const int e = eb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
                            const int tl = wt * WN + ni * 32 + l32 - zp * ZROWS;
                            if (e < E) {
                                float v = acc2[eb][ni][i];
                                if (pass == 0) {
                                    if (b2 && !split) v += bf16_bits_to_f32(b2[(long long)layer * E + e]);
                                } else {
                                    v = zs[tl * ZP + e] + v;
                                }
                                zs[tl * ZP + e] = v;
                            }
                        }
            }
            __syncthreads();
        }
    };
    // zs -> idx, probs (and logits) for the same rows
    auto finish_rows = [&](int zp) {
        const int tbase = t0 + zp * ZROWS;
        if (logits) {
            for (int i = tid; i < ZROWS * E; i += C::THREADS) {
                const int tl = i / E, e = i - tl * E;
                if (tbase + tl < T) logits[((long long)layer * T + tbase + tl) * E + e] = zs[tl * ZP + e];
            }
        }
        const int tl = tid / ZG, gg = tid % ZG;
        // the lanes of a group take the same branch (same token)
        if (tbase + tl < T) {
            const long long row = (long long)layer * T + tbase + tl;
            const EpilogueOut eo{prob_mode, margin ? margin + row : nullptr, counts ? cnt_lds : nullptr};
            row_softmax_topk_upto16<ZG>(zs + tl * ZP, E, k, gg, idx + row * k, probs + row * k, eo);
        }
        __syncthreads();
    };

    if (!split) {
#pragma unroll 1
        for (int zp = 0; zp < BM / ZROWS; ++zp) {
            regs_to_lds(zp);
            finish_rows(zp);
        }
        flush_counts();
        return;
    }

    // r is split over `groups` workgroups: park this group's score tile in the
    // workspace as zpart[tile][group][token][expert]; the workgroup that arrives
    // last (ticket counter, release/acquire fences) adds the groups in ascending
    // order -- a fixed order, whoever is last -- and finishes the rows.
    float* zmine = zpart + ((long long)(tile_id - split_tile0) * groups + cg) * BM * E;
#pragma unroll 1
    for (int zp = 0; zp < BM / ZROWS; ++zp) {
        regs_to_lds(zp);
        for (int i = tid; i < ZROWS * E; i += C::THREADS) {
            const int tl = i / E, e = i - tl * E;
            if (t0 + zp * ZROWS + tl < T) zmine[(long long)(zp * ZROWS + tl) * E + e] = zs[tl * ZP + e];
        }
        __syncthreads();
    }
    // One thread publishes for the workgroup: the barrier orders every thread's
    // stores before its device-scope release fence, and its acquire fence before
    // every thread's later loads (one L2 write-back / invalidate per workgroup,
    // not one per thread).
    __syncthreads();
    int* flag = (int*)smem_raw;
    if (tid == 0) {
        __threadfence();
        const int ticket = atomicAdd(&tickets[tile_id - split_tile0], 1);
        if (ticket == groups - 1) __threadfence();
        *flag = ticket;
    }
    __syncthreads();
    const bool last = (*flag == groups - 1);
    __syncthreads();
    if (!last) return;
    const float* zall = zpart + (long long)(tile_id - split_tile0) * groups * BM * E;
#pragma unroll 1
    for (int zp = 0; zp < BM / ZROWS; ++zp) {
        if (t0 + zp * ZROWS >= T) break;                      // no tokens left in this tile (uniform)
        for (int i = tid; i < ZROWS * E; i += C::THREADS) {
            const int tl = i / E, e = i - tl * E;
            if (t0 + zp * ZROWS + tl >= T) continue;
            const float* src = zall + (long long)(zp * ZROWS + tl) * E + e;
            float v = 0.0f;
            for (int q0 = 0; q0 < groups; q0 += 8) {          // eight loads in flight, added in ascending order
                float part[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) part[u] = (q0 + u < groups) ? src[(long long)(q0 + u) * BM * E] : 0.0f;
#pragma unroll
                for (int u = 0; u < 8; ++u) v += part[u];
            }
            if (b2) v += bf16_bits_to_f32(b2[(long long)layer * E + e]);
            zs[tl * ZP + e] = v;
        }
        __syncthreads();
        finish_rows(zp);
    }
    flush_counts();
}

__global__ void prefill_clear_tickets(int* tickets, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) tickets[i] = 0;
}

// Configurations (all 8 waves and one workgroup per CU except Small).  The 160 KB of
// LDS hold the stages and, behind them, the chunk's W2 slice (E rounded up to 32 rows x
// BN hidden units x 2 bytes):
//   Big       256 x 256 tile, waves 2 x 4 (128 units x 64 tokens each: 0.75 LDS fragment reads per
//             matrix instruction, the fewest bytes per flop through the CU's vector memory path),
//             E <= 64; four 32-wide stages of 32 KB + 32 KB slice.
//   BigDeep   the same tile in two 64-wide stages (64 KB each) + 32 KB slice: half as many barriers
//             per flop, measured +3% at d = 4096 and no better at d = 2048.
//   BigWide   the 256 x 256 tile with the 8 waves side by side along tokens (256 units x 32 tokens
//             each: 128 + 64 accumulators per lane) for 64 < E <= 128; three 32-wide stages + 64 KB
//             slice.  Measured on the Qwen3-30B-A3B shape: 934 TFLOP/s against 791 for Mid.
//   Mid       256 tokens x 128 hidden units, waves 2 x 4 (64 units x 64 tokens each, 128 score
//             accumulators per lane), 64 < E <= 128 when r is not a multiple of 256; five 32-wide
//             stages of 24 KB + 32 KB slice.
//   MidWide   the same tile with the waves side by side along tokens, which halves the score
//             accumulators per lane (E up to 256) at 1.25 fragment reads per matrix instruction;
//             four stages of 24 KB + 64 KB slice.
//   Small     128 x 128, 4 waves, two workgroups per CU (4 x 16 KB + 16 KB slice each): short inputs
//             and any r that is a multiple of 128.  SmallWide: the same for E > 64 (64 KB slice).
typedef PfCfg<256, 256, 32, 4, 2, 4, 1> CfgBig;
typedef PfCfg<256, 256, 64, 2, 2, 4, 1> CfgBigDeep;      // long rows (d >= 4096): half as many barriers per flop
typedef PfCfg<256, 128, 32, 5, 2, 4, 1> CfgMid;
typedef PfCfg<256, 256, 32, 3, 1, 8, 1> CfgBigWide;      // 64 < E <= 128, r a multiple of 256
typedef PfCfg<256, 128, 32, 4, 1, 8, 1> CfgMidWide;
typedef PfCfg<128, 128, 32, 4, 2, 2, 2> CfgSmall;
typedef PfCfg<128, 128, 32, 4, 1, 4, 1> CfgSmallWide;

template <class C, int EB32>
static size_t cfg_lds_bytes(int E)
{
    // score tile of the epilogue, then E activation counters
    const size_t z = sizeof(float) * (size_t)PfZRows<C, EB32>::value * (size_t)(E + 1) + sizeof(int32_t) * (size_t)E;
    // main loop: the stages, then the W2 slice (32 * EB32 rows of BN hidden units)
    const size_t loop = (size_t)C::TILE_BYTES + (C::W2L ? (size_t)EB32 * 32 * C::BN * 2 : 0);
    return z > loop ? z : loop;
}

bool prefill_supported(const PredictArgs& a)
{
    // the copy offsets are 32-bit byte offsets into one layer's W1 and x
    const int list = a.k + ((a.margin && a.k < a.E) ? 1 : 0);     // the epilogue keeps sorted lists of up to 16
    return a.dtype == 1 && a.T >= 1 && a.d % 32 == 0 && a.r % 128 == 0 && a.E <= 256 && list <= 16 &&
           (long long)a.r * a.d * 2 < (1ll << 31) && ((long long)a.T + 256) * a.d * 2 < (1ll << 31);
}

// How many workgroups share one token tile (each takes r / BN / groups chunks
// and the last one to finish adds their score tiles).
//  * Fewer tiles than CU slots (short inputs, down to a single tile per layer,
//    where the kernel is a weight-streaming problem): split until there are
//    about one and a half workgroups per CU, so that the whole chip pulls on
//    HBM.
//  * Many tiles: splitting lets the workgroups of one XCD share a token tile
//    through L2 instead of each pulling its own from far memory once per chunk
//    (measured: 3.3x fewer bytes fetched past L2 at 8 groups), but every extra
//    group costs a pipeline fill, a score tile written and re-read, and a
//    device-scope fence.  Measured on the paper's shapes it pays only when the
//    token tile is large (d >= 4096: 2 MB per tile), and then with two groups.
template <class C>
static int prefill_groups(const PredictArgs& a)
{
    const int NC = a.r / C::BN;
    const long long tiles = (long long)((a.T + C::BM - 1) / C::BM) * a.L;
    if (tiles < 256) {
        int g = 1;
        while (g < NC && (tiles * g < 384 || NC % g != 0)) ++g;
        return g;
    }
    if (NC % 2 != 0) return 1;
    return ((long long)a.d * C::BM * 2 >= (2ll << 20)) ? 2 : 1;
}

// How a launch is laid out: `main_tiles` token tiles with `main_groups` workgroups each, then
// `tail_tiles` with `tail_groups` each.  With whole-tile workgroups (main_groups = 1) the tiles beyond the
// last full round of 256 would keep a fraction of the CUs busy for a whole tile's duration; where it pays
// they are cut along r into pieces short enough to fill every CU evenly, at the price of the score-tile
// exchange (measured, 2048 x 2048 layers of 16 tiles: 20 layers 842 -> 985 TFLOP/s, 24 layers 934 -> 1015;
// with 26 layers the tail of 160 tiles is too long for any cut to win and stays whole).
struct PfLayout {
    int main_tiles, main_groups, tail_tiles, tail_groups;
    int split_tile0, split_tiles, split_groups;              // the tiles that go through the workspace
};
template <class C>
static PfLayout cfg_layout(const PredictArgs& a)
{
    const int NC = a.r / C::BN;
    const int tiles = ((a.T + C::BM - 1) / C::BM) * a.L;
    PfLayout f{tiles, prefill_groups<C>(a), 0, 1, 0, 0, 1};
    if (f.main_groups > 1) {
        f.split_tiles = tiles;
        f.split_groups = f.main_groups;
        return f;
    }
    constexpr int CUS = 256;
    const int tail = tiles % CUS;
    if (tiles < CUS || tail == 0) return f;
    // Time of the tail in units of one whole-tile workgroup on a full chip, from measurements on 2048 x 2048
    // layers: uncut, the tail's workgroups run faster than on a full chip (the clock rises when CUs idle:
    // 0.62 for 64 tiles, 0.76 for 128, 0.92 for 160); cut g ways they take 1/g plus about 0.08 each (pipeline
    // fill, the score-tile exchange, and the XCD's workgroups no longer walking the same chunk of W1).
    int best = 1;
    double best_t = 0.55 + 0.40 * tail / CUS;
    for (int g = 2; g <= 8 && g <= NC; g *= 2) {
        if (NC % g != 0) continue;
        const double t = (double)((tail * g + CUS - 1) / CUS) * (1.0 / g + 0.08);
        if (t < best_t - 0.05) { best_t = t; best = g; }
    }
    if (best == 1) return f;
    f.main_tiles = tiles - tail;
    f.tail_tiles = tail;
    f.tail_groups = best;
    f.split_tile0 = f.main_tiles;
    f.split_tiles = tail;
    f.split_groups = best;
    return f;
}

template <class C>
static size_t cfg_workspace_bytes(const PredictArgs& a)
{
    const PfLayout f = cfg_layout<C>(a);
    if (f.split_tiles == 0) return 0;
    return (size_t)f.split_tiles * f.split_groups * C::BM * a.E * sizeof(float) +
           (((size_t)f.split_tiles * sizeof(int) + 15) / 16) * 16;
}

template <class C, int EB32>
static hipError_t launch_cfg(const PredictArgs& a)
{
    const int tiles = (a.T + C::BM - 1) / C::BM;
    const PfLayout f = cfg_layout<C>(a);
    const int main_wgs = f.main_tiles * f.main_groups, tail_wgs = f.tail_tiles * f.tail_groups;
    const size_t lds = cfg_lds_bytes<C, EB32>(a.E);
    float* zpart = nullptr;
    int* tickets = nullptr;
    if (f.split_tiles > 0) {
        zpart = (float*)a.workspace;
        tickets = (int*)((char*)a.workspace + (size_t)f.split_tiles * f.split_groups * C::BM * a.E * sizeof(float));
        hipLaunchKernelGGL(prefill_clear_tickets, dim3((f.split_tiles + 255) / 256), dim3(256), 0, a.stream, tickets,
                           f.split_tiles);
    }
    auto kern = prefill_kernel<C, EB32>;
    static LdsLimit limit;
    hipError_t err = ensure_lds_limit(limit, (const void*)kern, lds);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(kern, dim3(main_wgs + tail_wgs), dim3(C::THREADS), lds, a.stream, a.T, a.d, a.r, a.E, a.k, a.act,
                       tiles, main_wgs, f.main_groups, tail_wgs, f.tail_groups, f.split_tile0, a.r / C::BN,
                       a.x_stride, a.w1_stride, a.w2_stride, (const uint16_t*)a.x,
                       (const uint16_t*)a.W1, (const uint16_t*)a.W2, (const uint16_t*)a.b1,
                       (const uint16_t*)a.b2, a.idx, a.probs, a.logits, zpart, tickets, a.counts, a.prob_mode,
                       a.margin);
    return hipGetLastError();
}

// The large tiles pay off once they fill a good part of the 256 CUs; below
// that, more and smaller workgroups win.
static bool enough_large_tiles(const PredictArgs& a) { return (long long)((a.T + 255) / 256) * a.L >= 128; }

// 0: small, 1: small wide, 2: big, 3: mid, 4: big wide
static int pick_cfg(const PredictArgs& a)
{
    const bool large = enough_large_tiles(a);
    if (a.E <= 64) return (large && a.r % 256 == 0) ? 2 : 0;
    if (!large) return 1;
    return (a.E <= 128 && a.r % 256 == 0) ? 4 : 3;
}

template <class C>
static void cfg_plan(const PredictArgs& a, int* groups, int* cpg)
{
    const PfLayout f = cfg_layout<C>(a);
    *groups = f.main_groups;
    *cpg = a.r / C::BN / f.main_groups;
}

void prefill_plan(const PredictArgs& a, int* cfg, int* groups, int* chunks_per_group)
{
    *cfg = pick_cfg(a);
    switch (*cfg) {
    case 2: cfg_plan<CfgBig>(a, groups, chunks_per_group); break;
    case 3: cfg_plan<CfgMid>(a, groups, chunks_per_group); break;
    case 4: cfg_plan<CfgBigWide>(a, groups, chunks_per_group); break;
    case 1: cfg_plan<CfgSmallWide>(a, groups, chunks_per_group); break;
    default: cfg_plan<CfgSmall>(a, groups, chunks_per_group); break;
    }
}

size_t prefill_workspace_bytes(const PredictArgs& a)
{
    switch (pick_cfg(a)) {
    case 2: return cfg_workspace_bytes<CfgBig>(a);
    case 3: return cfg_workspace_bytes<CfgMid>(a);
    case 4: return cfg_workspace_bytes<CfgBigWide>(a);
    case 1: return cfg_workspace_bytes<CfgSmallWide>(a);
    default: return cfg_workspace_bytes<CfgSmall>(a);
    }
}

hipError_t launch_predict_prefill(const PredictArgs& a)
{
    switch (pick_cfg(a)) {
    case 2:
        if (a.d >= 4096 && a.d % 64 == 0) return a.E <= 32 ? launch_cfg<CfgBigDeep, 1>(a) : launch_cfg<CfgBigDeep, 2>(a);
        return a.E <= 32 ? launch_cfg<CfgBig, 1>(a) : launch_cfg<CfgBig, 2>(a);
    case 3: return a.E <= 128 ? launch_cfg<CfgMid, 4>(a) : launch_cfg<CfgMidWide, 8>(a);
    case 4: return launch_cfg<CfgBigWide, 4>(a);
    case 1: return a.E <= 128 ? launch_cfg<CfgSmallWide, 4>(a) : launch_cfg<CfgSmallWide, 8>(a);
    default: return a.E <= 32 ? launch_cfg<CfgSmall, 1>(a) : launch_cfg<CfgSmall, 2>(a);
    }
}

}  // namespace paep

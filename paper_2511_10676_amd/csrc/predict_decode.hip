// Decode-shaped predictor (T <= 64 tokens per layer), bf16 storage.
//
// At a handful of tokens the predictor is a weight-streaming problem: every
// byte of W1 (r x d) and W2 (E x r) is needed once and the arithmetic per byte
// is tiny, so the kernels are organised around reading the weights from HBM
// exactly once, coalesced, with many loads in flight and nothing in the way.
// One predictor belongs to one layer (paper section 4.2) and a layer is only
// ~8 MB, so all layers of a call are spread over one grid.
//
// Kernel 1 (partial): the inner width r is cut into slices; workgroup (slice,
// layer) owns W1[slice rows, :] and W2[:, slice], forms h^T[slice, T] with
// v_mfma_f32_16x16x32_bf16, rounds it to bf16 (bias and activation applied)
// and multiplies it by the W2 column slice with the same instruction; that is
// the slice's contribution to the scores and goes to the workspace as fp32
// partial[layer][slice][t][e].  Two forms:
//   rows   (r a multiple of 128) slices of 128 hidden units, eight waves that
//          split the ROWS: a wave streams its 16 rows over the whole of d into
//          registers and all waves take the tokens from LDS, where the
//          workgroup puts them once (decode_rows_kernel below).
//   d-split  slices of 64 hidden units, four waves that split d into quarters,
//          weights and tokens both straight into registers, the four partial
//          sums added in LDS wave after wave (decode_partial_kernel).
// In both a lane reads 16 contiguous bytes of one row, four neighbouring lanes
// 64 contiguous bytes, and a lane permutation puts the fragment into the
// A-operand layout.
//
// Kernel 2 (finalize): one wave per token adds the slices in ascending order
// (fixed order, so the result is reproducible; up to 32 loads in flight), adds b2, and runs softmax and
// top-k (eq. 1 and eq. 4) in registers with wave shuffles.
#include <type_traits>

#include "paep_device.h"
#include "paep_internal.h"

namespace paep {

static constexpr int DEC_THREADS = 256;
static constexpr int RS = 64;            // hidden units per workgroup
static constexpr int RB = RS / 16;       // 16-row blocks per workgroup
static constexpr int HPAD = 8;

template <int V> using IC = std::integral_constant<int, V>;
template <int N, class F> __device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(IC<N - 1>{});
    }
}

// TB: 16-token blocks (T <= 16 * TB); U: k-steps per load batch; NBUF: load
// batches in the register ring (NBUF - 1 are in flight while one is multiplied).
template <int TB, int U, int NBUF>
__global__ __launch_bounds__(DEC_THREADS) void decode_partial_kernel(
    int T, int d, int r, int E, int act, int S, int total_wgs, long long xs_, long long w1s, long long w2s,
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ W1, const uint16_t* __restrict__ W2,
    const uint16_t* __restrict__ b1, float* __restrict__ partial)
{
    constexpr int TP = 16 * TB;
    __shared__ __attribute__((aligned(16))) float hsum[RB * TB * 64 * 4];          // partial h, summed wave after wave
    __shared__ __attribute__((aligned(16))) uint16_t ht[TP * (RS + HPAD)];        // h as bf16, [token][unit]

    // Work item = (layer, slice), slice fastest.  Workgroups are dealt round-robin
    // to the 8 XCDs; remap so that each XCD walks a contiguous range of items: the
    // workgroups an XCD runs at the same time are then neighbouring slices of one
    // layer and find that layer's tokens in the XCD's L2, and a layer's tokens are
    // fetched from memory by one or two XCDs instead of all eight.
    int item = blockIdx.x;
    {
        const int per = total_wgs / 8, rem = total_wgs % 8;
        const int xcd = item % 8, slot = item / 8;
        item = xcd * per + (xcd < rem ? xcd : rem) + slot;
    }
    const int layer = item / S, slice = item - layer * S;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 15, kg = lane >> 4;
    const uint16_t* xl = x + (long long)layer * xs_;
    const uint16_t* W1l = W1 + (long long)layer * w1s;
    const uint16_t* W2l = W2 + (long long)layer * w2s;

    // this wave's quarter of d
    const int kq = d / 4, k0 = wave * kq;
    const int nsteps = kq / 32;                               // MFMA k-steps per wave
    // Which 16 bytes a lane fetches of a 16-row x 64-byte fragment.  The matrix instruction wants lane
    // (m, kg) to hold row m, bytes 16*kg..; fetched that way, neighbouring lanes touch different rows and
    // every lane is a separate 16-byte access to the vector cache.  So lane l fetches row l/4, bytes
    // 16*(l%4).. instead -- four neighbouring lanes form one 64-byte access -- and the fragment is put
    // into the instruction's layout afterwards by a fixed lane permutation (lane (m, kg) takes from lane
    // 4*m + kg; ds_bpermute moves registers between lanes without touching LDS memory).  Measured on
    // the 26 x (2048 x 2048) bank: -6% time at 1 token, -14% at 64.
    const int lrow = lane >> 2, lchunk = lane & 3;
    const int perm_src = (4 * m + kg) * 4;                   // byte address for ds_bpermute
    const uint16_t* arow = W1l + (long long)(slice * RS + lrow) * d + k0 + lchunk * 8;   // + rb*16*d + step*32
    const uint16_t* brow = xl + (long long)lrow * d + k0 + lchunk * 8;                  // + tb*16*d + step*32
    bool tok_ok[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) tok_ok[tb] = (tb * 16 + lrow) < T;
    auto to_mfma_layout = [&](const u32x4& f) {
        return u32x4{(uint32_t)__builtin_amdgcn_ds_bpermute(perm_src, (int)f[0]),
                          (uint32_t)__builtin_amdgcn_ds_bpermute(perm_src, (int)f[1]),
                          (uint32_t)__builtin_amdgcn_ds_bpermute(perm_src, (int)f[2]),
                          (uint32_t)__builtin_amdgcn_ds_bpermute(perm_src, (int)f[3])};
    };

    // W2 fragments of this wave's first expert blocks, requested now and used at the very end
    constexpr int NPF = 2;
    const int EB = (E + 15) / 16;
    u32x4 w2pf[NPF][RS / 32];
#pragma unroll
    for (int j = 0; j < NPF; ++j) {
        const int e_row = (wave + 4 * j) * 16 + m;
#pragma unroll
        for (int s = 0; s < RS / 32; ++s) {
            w2pf[j][s] = u32x4{0u, 0u, 0u, 0u};
            if (e_row < E) w2pf[j][s] = *(const u32x4*)(W2l + (long long)e_row * r + slice * RS + s * 32 + kg * 8);
        }
    }

    f32x4 acc[RB][TB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) acc[rb][tb] = f32x4{0.f, 0.f, 0.f, 0.f};

    u32x4 fa[NBUF][U][RB], fb[NBUF][U][TB];
    auto load_batch = [&](auto buf_c, int step0) {
        constexpr int buf = decltype(buf_c)::value;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int off = (step0 + u) * 32;
            const bool live = step0 + u < nsteps;             // wave-uniform; steps past the end multiply zeros
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                fa[buf][u][rb] = u32x4{0u, 0u, 0u, 0u};
                if (live) fa[buf][u][rb] = *(const u32x4*)(arow + (long long)rb * 16 * d + off);
            }
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                fb[buf][u][tb] = u32x4{0u, 0u, 0u, 0u};
                if (live && tok_ok[tb]) fb[buf][u][tb] = *(const u32x4*)(brow + (long long)tb * 16 * d + off);
            }
        }
    };
    auto mma_batch = [&](auto buf_c) {
        constexpr int buf = decltype(buf_c)::value;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            u32x4 pa[RB], pb[TB];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) pa[rb] = to_mfma_layout(fa[buf][u][rb]);
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) pb[tb] = to_mfma_layout(fb[buf][u][tb]);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int tb = 0; tb < TB; ++tb)
                    acc[rb][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8, pa[rb]), __builtin_bit_cast(bf16x8, pb[tb]),
                        acc[rb][tb], 0, 0, 0);
        }
    };

    // Ring of NBUF register batches: batch i + NBUF - 1 is requested, then batch i is multiplied,
    // so NBUF - 1 batches of loads are in flight behind the arithmetic.
    static_for<NBUF - 1>([&](auto b_c) { load_batch(b_c, decltype(b_c)::value * U); });
    for (int s0 = 0; s0 < nsteps; s0 += NBUF * U) {
        static_for<NBUF>([&](auto b_c) {
            constexpr int b = decltype(b_c)::value;
            load_batch(IC<(b + NBUF - 1) % NBUF>{}, s0 + (b + NBUF - 1) * U);
            if (s0 + b * U < nsteps) mma_batch(b_c);          // wave-uniform
        });
    }

    // acc[rb][tb][i] = partial h[token tb*16 + m][unit slice*RS + rb*16 + 4*kg + i] over this wave's quarter of d.
    // The four partial sums are added in LDS wave after wave (w0 + w1 + w2 + w3, a fixed order) in one buffer.
#pragma unroll 1
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int tb = 0; tb < TB; ++tb) {
                    f32x4* slot = (f32x4*)(&hsum[((rb * TB + tb) * 64 + lane) * 4]);
                    f32x4 v = acc[rb][tb];
                    if (w > 0) {
                        const f32x4 o = *slot;
#pragma unroll
                        for (int i = 0; i < 4; ++i) v[i] = o[i] + v[i];
                    }
                    *slot = v;
                }
        }
        __syncthreads();
    }
    for (int q = tid; q < RB * TB * 64; q += DEC_THREADS) {
        const int ln = q & 63, blk = q >> 6, tb = blk % TB, rb = blk / TB;
        const int unit = rb * 16 + 4 * (ln >> 4), tok = tb * 16 + (ln & 15);
        const f32x4 v = *(const f32x4*)(&hsum[q * 4]);
        float h[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float t = v[i];
            if (b1) t += bf16_bits_to_f32(b1[(long long)layer * r + slice * RS + unit + i]);
            t = round_to_bf16(t);
            if (act != 0) t = round_to_bf16(apply_act(t, act));
            h[i] = t;
        }
        *(u32x2*)(ht + tok * (RS + HPAD) + unit) = u32x2{pack_bf16x2(h[0], h[1]), pack_bf16x2(h[2], h[3])};
    }
    __syncthreads();

    // scores of this slice: z^T[e, t] = W2[e, slice] . h^T[slice, t]
    auto score_block = [&](int eb, const u32x4 (&wfrag)[RS / 32]) {
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
                if (eb * 16 + 4 * kg + 3 < E) {
                    *(f32x4*)dst = z;
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (eb * 16 + 4 * kg + i < E) dst[i] = z[i];
                }
            }
        }
    };
#pragma unroll
    for (int j = 0; j < NPF; ++j)
        if (wave + 4 * j < EB) score_block(wave + 4 * j, w2pf[j]);
    for (int eb = wave + 4 * NPF; eb < EB; eb += 4) {
        const int e_row = eb * 16 + m;
        u32x4 wfrag[RS / 32];
#pragma unroll
        for (int s = 0; s < RS / 32; ++s) {
            wfrag[s] = u32x4{0u, 0u, 0u, 0u};
            if (e_row < E) wfrag[s] = *(const u32x4*)(W2l + (long long)e_row * r + slice * RS + s * 32 + kg * 8);
        }
        score_block(eb, wfrag);
    }
}

// The row-split form.  What a CU's vector memory path can have in flight, not HBM, is what the d-split kernel
// waits for, and tokens take their share of it: every 64-row slice fetches all T tokens again (at 64 tokens
// as many bytes as the slice itself), and whether they come from L2 or from the CU's own cache makes no
// difference to the time (measured).  Here a workgroup takes 128 hidden units, so the tokens are fetched once
// per 128 rows, and the waves divide the rows instead of d: wave w owns rows 16w..16w+15 of the slice over
// the whole of d and streams them into registers; all eight waves take the tokens from LDS, where each stage
// of 128 columns is put once per workgroup by direct global -> LDS copies (a ring of two or three stages, one
// workgroup barrier per stage: with two workgroups on a CU one stage of requests ahead per wave already
// over-fills the memory pipeline and deeper rings measured 2-3 % slower; with one workgroup per CU two
// stages ahead are 5-9 % faster).  A wave's accumulators are the finished h of its rows: nothing to add up
// across waves.  Token row t of a stage is 256 bytes = 16 chunks of 16 bytes, chunk c in slot c ^ (t % 16)
// (chosen on the global side of the copy), so that the 16 lanes of a fragment read, which take the same
// chunk of 16 different tokens, fall into 16 different slots.  Measured on 26 layers of 2048 x 2048 against
// the d-split kernel: 53.8 -> 49.8 us at 1 token, 58.7 -> 51.2 at 16, 79.7 -> 57.6 at 64.
static constexpr int RW_WAVES = 8;
static constexpr int RW_RS = 16 * RW_WAVES;          // hidden units per workgroup
static constexpr int RW_KST = 128;                   // columns of d per stage

typedef void __attribute__((address_space(3)))* lds_ptr_t;
// s_waitcnt immediate that waits for vmcnt <= n and nothing else (gfx9 encoding)
#define PAEP_DEC_VMCNT(n) ((((n) & 0xF) | (((n) >> 4) << 14)) | 0x0F70)

// TB: 16-token blocks held in LDS, 2 (T <= 32) or 4; RW_NSTG: stages in the ring, 2 or 3
template <int TB, int RW_NSTG>
__global__ __launch_bounds__(RW_WAVES * 64, 4) void decode_rows_kernel(
    int T, int d, int r, int E, int act, int S, int total_wgs, long long xs_, long long w1s, long long w2s,
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ W1, const uint16_t* __restrict__ W2,
    const uint16_t* __restrict__ b1, float* __restrict__ partial)
{
    constexpr int TP = 16 * TB;
    constexpr int STAGE_BYTES = TP * RW_KST * 2;
    constexpr int XJ = TP / 4 / RW_WAVES;            // copy instructions per wave and stage (4 token rows each)
    constexpr int KS = RW_KST / 32;                  // MFMA k-steps per stage
    static_assert(XJ * 4 * RW_WAVES == TP, "token rows divide among the waves");
    extern __shared__ __attribute__((aligned(16))) unsigned char dsmem[];   // the ring; h (bf16) afterwards
    uint16_t* ht = (uint16_t*)dsmem;                                       // [token][unit], TP x (RW_RS + HPAD)
    static_assert(TP * (RW_RS + HPAD) * 2 <= RW_NSTG * STAGE_BYTES, "h fits in the ring");

    int item = blockIdx.x;
    {
        const int per = total_wgs / 8, rem = total_wgs % 8;
        const int xcd = item % 8, slot = item / 8;
        item = xcd * per + (xcd < rem ? xcd : rem) + slot;
    }
    const int layer = item / S, slice = item - layer * S;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 15, kg = lane >> 4;
    const uint16_t* xl = x + (long long)layer * xs_;
    const uint16_t* W1l = W1 + (long long)layer * w1s;
    const uint16_t* W2l = W2 + (long long)layer * w2s;
    const int NST = d / RW_KST;

    // token copies: instruction q = wave * XJ + j moves token rows 4q..4q+3 of a stage; lane l supplies the
    // chunk that belongs in slot l % 16 of row 4q + l / 16.  Rows past T lie outside the resource: zeros.
    const __amdgpu_buffer_rsrc_t rsrc_x =
        __builtin_amdgcn_make_buffer_rsrc((void*)xl, 0, (int)((long long)T * d * 2), 0x00020000);
    uint32_t xlane[XJ];
#pragma unroll
    for (int j = 0; j < XJ; ++j) {
        const int t = (wave * XJ + j) * 4 + (lane >> 4);
        const int c = (lane & 15) ^ (t & 15);
        xlane[j] = (uint32_t)(t * d + c * 8) * 2u;
    }
    auto issue_x = [&](int stage, int slot) {
#pragma unroll
        for (int j = 0; j < XJ; ++j)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_x, (lds_ptr_t)(dsmem + slot * STAGE_BYTES + (wave * XJ + j) * 1024),
                                                     16, (int)xlane[j], stage * RW_KST * 2, 0, 0);
    };
    // this wave's 16 rows of W1, fetched as in the kernel above (lane l: row l / 4, bytes 16 * (l % 4) of a
    // 64-byte k-step) and permuted into the A-operand layout
    const int lrow = lane >> 2, lchunk = lane & 3;
    const int perm_src = (4 * m + kg) * 4;
    // (buffer-addressed: base and bounds of the wave's 16 rows in scalar registers, a fixed 32-bit lane offset and
    // a scalar stage offset, so that no vector register is spent on addresses inside the loop)
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(W1l + (long long)(slice * RW_RS + wave * 16) * d), 0, 16 * d * 2, 0x00020000);
    const int wlane = (lrow * d + lchunk * 8) * 2;
    auto to_mfma_layout = [&](const u32x4& f) {
        return u32x4{(uint32_t)__builtin_amdgcn_ds_bpermute(perm_src, (int)f[0]),
                     (uint32_t)__builtin_amdgcn_ds_bpermute(perm_src, (int)f[1]),
                     (uint32_t)__builtin_amdgcn_ds_bpermute(perm_src, (int)f[2]),
                     (uint32_t)__builtin_amdgcn_ds_bpermute(perm_src, (int)f[3])};
    };
    u32x4 fa[RW_NSTG][KS];
    auto load_w = [&](auto buf_c, int stage) {
        constexpr int buf = decltype(buf_c)::value;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            fa[buf][ks] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, wlane + ks * 64, stage * (RW_KST * 2), 0));
    };

    // W2 fragments of this wave's first expert block, requested now and used at the very end
    const int EB = (E + 15) / 16;
    u32x4 w2pf[RW_RS / 32];
    {
        const int e_row = wave * 16 + m;
#pragma unroll
        for (int s = 0; s < RW_RS / 32; ++s) {
            w2pf[s] = u32x4{0u, 0u, 0u, 0u};
            if (e_row < E) w2pf[s] = *(const u32x4*)(W2l + (long long)e_row * r + slice * RW_RS + s * 32 + kg * 8);
        }
    }

    f32x4 acc[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) acc[tb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Stage s: its token copies and this wave's rows are requested RW_NSTG - 1 stages ahead, in that order, so
    // at the top of stage s only the requests of the RW_NSTG - 2 stages after it may still be in flight.  Past
    // the last stage the last one is requested again (into a slot nobody reads any more), which keeps that
    // count the same on every iteration.
    constexpr int WAIT_STAGE = PAEP_DEC_VMCNT((RW_NSTG - 2) * (XJ + KS));
    // Workgroups start at different columns and wrap around (the s-th stage a workgroup works on is columns
    // 128 * ((s + item) % NST) ..): all waves of the chip advance at about the same pace, and with a common
    // starting column the addresses in flight at any moment would differ only in bits 12 and up -- rows are a
    // power of two apart -- which lands them on a few memory channels for some placements of the weights
    // (measured: 58 us against 48 us for one of four identically shaped banks; the same 48 us for all four with
    // the rotation).  The order in which a workgroup adds up d is fixed by its position in the grid.
    const int rot = item % NST;
    auto column_stage = [&](int s) { return s + rot < NST ? s + rot : s + rot - NST; };
    static_for<RW_NSTG - 1>([&](auto b_c) {
        constexpr int b = decltype(b_c)::value;
        const int st = column_stage(b < NST ? b : NST - 1);
        issue_x(st, b);
        __builtin_amdgcn_sched_barrier(0);
        load_w(b_c, st);
        __builtin_amdgcn_sched_barrier(0);
    });
    for (int s0 = 0; s0 < NST; s0 += RW_NSTG) {
        static_for<RW_NSTG>([&](auto b_c) {
            constexpr int b = decltype(b_c)::value;
            const int s = s0 + b;
            if (s < NST) {                                        // uniform over the workgroup
                __builtin_amdgcn_s_waitcnt(WAIT_STAGE);           // this wave's part of stage s has landed
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_barrier();                     // everyone's has; and everyone is done with stage s - 1
                asm volatile("" ::: "memory");
                const int sn = column_stage(s + RW_NSTG - 1 < NST ? s + RW_NSTG - 1 : NST - 1);
                issue_x(sn, (b + RW_NSTG - 1) % RW_NSTG);
                __builtin_amdgcn_sched_barrier(0);
                load_w(IC<(b + RW_NSTG - 1) % RW_NSTG>{}, sn);
                __builtin_amdgcn_sched_barrier(0);
                const unsigned char* stage = dsmem + b * STAGE_BYTES;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    u32x4 pb[TB];
#pragma unroll
                    for (int tb = 0; tb < TB; ++tb)
                        pb[tb] = *(const u32x4*)(stage + (tb * 16 + m) * (RW_KST * 2) + (((ks * 4 + kg) ^ m) << 4));
                    const u32x4 pa = to_mfma_layout(fa[b][ks]);
#pragma unroll
                    for (int tb = 0; tb < TB; ++tb)
                        acc[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf16x8, pa), __builtin_bit_cast(bf16x8, pb[tb]), acc[tb], 0, 0, 0);
                }
            }
        });
    }
    // acc[tb][i] = h[token tb*16 + m][unit slice*RW_RS + wave*16 + 4*kg + i].  The ring is handed over to h once
    // every copy still in flight has landed and every wave has read its last fragments.
    __builtin_amdgcn_s_waitcnt(PAEP_DEC_VMCNT(0));
    __syncthreads();
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        const int unit = wave * 16 + 4 * kg, tok = tb * 16 + m;
        float h[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float t = acc[tb][i];
            if (b1) t += bf16_bits_to_f32(b1[(long long)layer * r + slice * RW_RS + unit + i]);
            t = round_to_bf16(t);
            if (act != 0) t = round_to_bf16(apply_act(t, act));
            h[i] = t;
        }
        *(u32x2*)(ht + tok * (RW_RS + HPAD) + unit) = u32x2{pack_bf16x2(h[0], h[1]), pack_bf16x2(h[2], h[3])};
    }
    __syncthreads();

    // scores of this slice: z^T[e, t] = W2[e, slice] . h^T[slice, t]; expert blocks dealt to the waves
    auto score_block = [&](int eb, const u32x4 (&wfrag)[RW_RS / 32]) {
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            f32x4 z = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < RW_RS / 32; ++s) {
                const u32x4 hv = *(const u32x4*)(ht + (tb * 16 + m) * (RW_RS + HPAD) + s * 32 + kg * 8);
                z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wfrag[s]),
                                                            __builtin_bit_cast(bf16x8, hv), z, 0, 0, 0);
            }
            const int t = tb * 16 + m;
            if (t < T) {
                float* dst = partial + (((long long)layer * S + slice) * T + t) * E + eb * 16 + 4 * kg;
                if (eb * 16 + 4 * kg + 3 < E) {
                    *(f32x4*)dst = z;
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (eb * 16 + 4 * kg + i < E) dst[i] = z[i];
                }
            }
        }
    };
    if (wave < EB) score_block(wave, w2pf);
    for (int eb = wave + RW_WAVES; eb < EB; eb += RW_WAVES) {
        const int e_row = eb * 16 + m;
        u32x4 wfrag[RW_RS / 32];
#pragma unroll
        for (int s = 0; s < RW_RS / 32; ++s) {
            wfrag[s] = u32x4{0u, 0u, 0u, 0u};
            if (e_row < E) wfrag[s] = *(const u32x4*)(W2l + (long long)e_row * r + slice * RW_RS + s * 32 + kg * 8);
        }
        score_block(eb, wfrag);
    }
}

// One wave per token row: lane l owns experts l, l+64, ...  The slice partials
// are summed in ascending slice order, 32 loads in flight at a time.
static constexpr int FIN_NV = 8;                          // experts per lane at most: E <= 512

template <int NV>                                         // experts per lane: E <= 64 * NV
__global__ __launch_bounds__(DEC_THREADS) void decode_finalize_kernel(
    int T, int E, int k, int S, int rows_total, const float* __restrict__ partial,
    const uint16_t* __restrict__ b2, int32_t* __restrict__ idx, float* __restrict__ probs,
    float* __restrict__ logits, int32_t* __restrict__ counts, int prob_mode, float* __restrict__ margin)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * (DEC_THREADS / 64) + (threadIdx.x >> 6);
    if (row >= rows_total) return;
    const int layer = row / T, t = row - layer * T;
    const long long sstride = (long long)T * E;
    const float* src = partial + ((long long)layer * S * T + t) * E;
    // all of a row's experts at once, CH slices per round: NV * CH loads in flight, added in ascending slice order
    constexpr int CH = (NV >= 8) ? 4 : 32 / NV;
    float z[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) z[v] = 0.0f;
    for (int s0 = 0; s0 < S; s0 += CH) {
        float p[NV][CH];
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int e = lane + 64 * v;
#pragma unroll
            for (int u = 0; u < CH; ++u) p[v][u] = (e < E && s0 + u < S) ? src[(long long)(s0 + u) * sstride + e] : 0.0f;
        }
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int u = 0; u < CH; ++u)
                if (s0 + u < S) z[v] += p[v][u];          // uniform; a skipped slice adds nothing, not even +0
    }
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int e = lane + 64 * v;
        if (e < E) {
            if (b2) z[v] += bf16_bits_to_f32(b2[(long long)layer * E + e]);
            if (logits) logits[(long long)row * E + e] = z[v];
        }
    }
    const EpilogueOut eo{prob_mode, margin ? margin + row : nullptr, counts ? counts + (long long)layer * E : nullptr};
    // one expert per lane: rank counting; more: k rounds of a wave-wide maximum (measured at 128 experts, k = 8:
    // 6.8 us against 9.6 us for rank counting at 48 rows, 11.6 against 17.7 at 3072 rows)
    if constexpr (NV == 1) wave_softmax_topk_rank<NV>(z, E, k, lane, idx + (long long)row * k, probs + (long long)row * k, eo);
    else                   wave_softmax_topk<NV>(z, E, k, lane, idx + (long long)row * k, probs + (long long)row * k, eo);
}

bool decode_supported(const PredictArgs& a)
{
    // each wave takes a quarter of d in k-steps of 32
    return a.dtype == 1 && a.T >= 1 && a.T <= 64 && a.r % 64 == 0 && a.d % 128 == 0 && a.E <= 64 * FIN_NV &&
           a.k <= 32;
}

size_t decode_workspace_bytes(const PredictArgs& a)
{
    return sizeof(float) * (size_t)a.L * (size_t)(a.r / RS) * (size_t)a.T * (size_t)a.E;
}

// r in whole slices of 128: the row-split kernel (measured against the d-split kernel at 1 token: 26 layers of
// 2048 x 2048 49.2 against 53.8 us, 32 layers of 1024 x 4096 56.0 against 57.5, 48 layers of 2048 x 2048 equal;
// at 32 and 64 tokens 10-27 % faster)
static bool decode_by_rows(const PredictArgs& a) { return a.r % RW_RS == 0; }

hipError_t launch_predict_decode(const PredictArgs& a)
{
    const bool rows_kernel = decode_by_rows(a);
    const int S = a.r / (rows_kernel ? RW_RS : RS);
    const int total = S * a.L;
    float* partial = (float*)a.workspace;
    const int TB = (a.T + 15) / 16;
    if (rows_kernel) {
#define PAEP_LAUNCH_ROWS(TBV, NSV)                                                                          \
        {                                                                                                   \
            constexpr size_t lds = (size_t)NSV * 16 * TBV * RW_KST * 2;                                     \
            static LdsLimit limit;                                                                          \
            const hipError_t e1 = ensure_lds_limit(limit, (const void*)decode_rows_kernel<TBV, NSV>, lds);  \
            if (e1 != hipSuccess) return e1;                                                                \
            hipLaunchKernelGGL((decode_rows_kernel<TBV, NSV>), dim3(total), dim3(RW_WAVES * 64), lds, a.stream, \
                               a.T, a.d, a.r, a.E, a.act, S, total, a.x_stride, a.w1_stride, a.w2_stride,   \
                               (const uint16_t*)a.x, (const uint16_t*)a.W1, (const uint16_t*)a.W2,          \
                               (const uint16_t*)a.b1, partial);                                             \
        }
        // fewer than one and a half workgroups per CU: a deeper ring
        const bool deep = total < 384;
        if (TB <= 2) { if (deep) PAEP_LAUNCH_ROWS(2, 3) else PAEP_LAUNCH_ROWS(2, 2) }
        else         { if (deep) PAEP_LAUNCH_ROWS(4, 3) else PAEP_LAUNCH_ROWS(4, 2) }
#undef PAEP_LAUNCH_ROWS
    } else {
#define PAEP_LAUNCH_DEC(TBV, UV, NBV)                                                                       \
    hipLaunchKernelGGL((decode_partial_kernel<TBV, UV, NBV>), dim3(total), dim3(DEC_THREADS), 0, a.stream,  \
                       a.T, a.d, a.r, a.E, a.act, S, total, a.x_stride, a.w1_stride, a.w2_stride,           \
                       (const uint16_t*)a.x, (const uint16_t*)a.W1, (const uint16_t*)a.W2,                  \
                       (const uint16_t*)a.b1, partial)
    switch (TB) {
    // k-steps per load batch and batches in the ring, by measurement on 26 layers of 2048 x 2048:
    // two k-steps per batch while the registers allow three waves per SIMD, one with a deeper ring beyond
    case 1: PAEP_LAUNCH_DEC(1, 2, 2); break;
    case 2: PAEP_LAUNCH_DEC(2, 2, 2); break;
    case 3: PAEP_LAUNCH_DEC(3, 1, 3); break;
    default: PAEP_LAUNCH_DEC(4, 1, 3); break;
    }
#undef PAEP_LAUNCH_DEC
    }
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    const int rows = a.L * a.T;
    const int rows_per_wg = DEC_THREADS / 64;
#define PAEP_LAUNCH_FIN(NVV)                                                                                \
    hipLaunchKernelGGL(decode_finalize_kernel<NVV>, dim3((rows + rows_per_wg - 1) / rows_per_wg), dim3(DEC_THREADS), \
                       0, a.stream, a.T, a.E, a.k, S, rows, partial, (const uint16_t*)a.b2, a.idx, a.probs,          \
                       a.logits, a.counts, a.prob_mode, a.margin)
    if (a.E <= 64)       PAEP_LAUNCH_FIN(1);
    else if (a.E <= 128) PAEP_LAUNCH_FIN(2);
    else if (a.E <= 256) PAEP_LAUNCH_FIN(4);
    else                 PAEP_LAUNCH_FIN(8);
#undef PAEP_LAUNCH_FIN
    return hipGetLastError();
}

}  // namespace paep

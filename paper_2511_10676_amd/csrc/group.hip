// Per-expert grouping of the selected expert ids: histogram, device-wide
// exclusive scan, stable index compaction (a counting sort by expert id).
// This produces the prefetch list that the paper's workflow (section 4.2,
// third stage) derives from the selection: which experts are needed and which
// tokens need each of them.
//
// Up to FUSED_MAX_ITEMS selections per layer (and as long as the lists fit in
// LDS beside the histograms), one launch does all of it out of LDS
// (group_fused_kernel): a layer is cut into P parts, one workgroup each.  The
// workgroups of a layer do not talk to each other: every one of them counts
// the WHOLE layer (counting is the cheap phase, one LDS atomic per selection),
// so each knows the layer's offsets and how many selections of every expert
// lie before its own part, and then scatters only its own part (the expensive
// phase).  No workspace, no second launch, no waiting.  Longer layers take
// three launches, all layers of a call batched on gridDim.y:
//   hist     every wave owns WAVE_ITEMS consecutive flat positions and counts
//            them per expert in its own LDS histogram, then stores that
//            histogram row to the workspace: hist[layer][wave_chunk][E + 1]
//            (slot E counts ids outside [0, E)).
//   scan     one workgroup per layer turns each expert's column of that
//            matrix into running sums (the base of every chunk inside the
//            expert's group), yielding counts; a block scan over experts gives
//            offsets; a second scan compacts the non-empty experts into the
//            active list.
//   scatter  every wave revisits its positions in order, 64 at a time: lanes
//            holding the same expert find each other with ballots over the id
//            bits, take consecutive slots from the wave's LDS cursor for that
//            expert, and write their position.  Order inside a group is
//            ascending position because chunks, batches and lanes are all
//            visited in ascending order.
#include "paep_internal.h"

namespace paep {

static constexpr int GROUP_THREADS = 256;
static constexpr int GROUP_WAVES = GROUP_THREADS / 64;
static constexpr int WAVE_ITEMS = 1024;                 // positions per wave
static constexpr int BLOCK_ITEMS = WAVE_ITEMS * GROUP_WAVES;
static constexpr int MAX_E = 1024;

static inline int wave_chunks(long long n) { return (int)((n + WAVE_ITEMS - 1) / WAVE_ITEMS); }
static inline int block_chunks(long long n) { return (int)((n + BLOCK_ITEMS - 1) / BLOCK_ITEMS); }

__global__ __launch_bounds__(GROUP_THREADS) void group_hist_kernel(
    const int32_t* __restrict__ idx, int n, int E, int nwc, int32_t* __restrict__ hist)
{
    __shared__ int32_t lh[GROUP_WAVES][MAX_E + 1];
    const int layer = blockIdx.y, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int e = lane; e <= E; e += 64) lh[wave][e] = 0;
    __syncthreads();
    const int wc = blockIdx.x * GROUP_WAVES + wave;
    const long long base = (long long)wc * WAVE_ITEMS;
    const int32_t* src = idx + (long long)layer * n;
    for (int i = lane; i < WAVE_ITEMS; i += 64) {
        const long long p = base + i;
        if (p < n) {
            const int32_t e = src[p];
            atomicAdd(&lh[wave][(e >= 0 && e < E) ? e : E], 1);
        }
    }
    __syncthreads();
    if (wc < nwc) {
        int32_t* dst = hist + ((long long)layer * nwc + wc) * (E + 1);
        for (int e = lane; e <= E; e += 64) dst[e] = lh[wave][e];
    }
}

// exclusive scan of one int per thread over the 256-thread block
__device__ __forceinline__ int block_exclusive_scan(int v, int* total, int* buf)
{
    const int tid = threadIdx.x;
    buf[tid] = v;
    __syncthreads();
    for (int off = 1; off < GROUP_THREADS; off <<= 1) {
        const int add = (tid >= off) ? buf[tid - off] : 0;
        __syncthreads();
        buf[tid] += add;
        __syncthreads();
    }
    const int incl = buf[tid];
    *total = buf[GROUP_THREADS - 1];
    __syncthreads();
    return incl - v;
}

__global__ __launch_bounds__(GROUP_THREADS) void group_scan_kernel(
    int E, int nwc, int32_t* __restrict__ hist, int32_t* __restrict__ counts,
    int32_t* __restrict__ offsets, int32_t* __restrict__ active, int32_t* __restrict__ n_active,
    int32_t* __restrict__ n_invalid)
{
    __shared__ int buf[GROUP_THREADS];
    const int layer = blockIdx.x, tid = threadIdx.x;
    int32_t* h = hist + (long long)layer * nwc * (E + 1);
    // thread owns experts e = tid*per .. tid*per + per - 1 (consecutive, so that
    // the block scan over threads is a scan over experts)
    const int per = (E + GROUP_THREADS - 1) / GROUP_THREADS;   // <= 4
    int cnt[MAX_E / GROUP_THREADS];
    int mine = 0, mine_active = 0;
#pragma unroll
    for (int q = 0; q < MAX_E / GROUP_THREADS; ++q) {
        cnt[q] = 0;
        const int e = tid * per + q;
        if (q < per && e < E) {
            int run = 0;
            for (int wc0 = 0; wc0 < nwc; wc0 += 16) {       // 16 loads in flight, then their running sums
                int c[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) c[u] = (wc0 + u < nwc) ? h[(long long)(wc0 + u) * (E + 1) + e] : 0;
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    if (wc0 + u < nwc) h[(long long)(wc0 + u) * (E + 1) + e] = run;   // chunk's base inside the group
                    run += c[u];
                }
            }
            cnt[q] = run;
            counts[(long long)layer * E + e] = run;
            mine += run;
            mine_active += (run > 0);
        }
    }
    int total, total_active;
    int off = block_exclusive_scan(mine, &total, buf);
    int aoff = block_exclusive_scan(mine_active, &total_active, buf);
    int32_t* offs = offsets + (long long)layer * (E + 1);
    int32_t* act = active + (long long)layer * E;
#pragma unroll
    for (int q = 0; q < MAX_E / GROUP_THREADS; ++q) {
        const int e = tid * per + q;
        if (q < per && e < E) {
            offs[e] = off;
            off += cnt[q];
            if (cnt[q] > 0) act[aoff++] = e;
        }
    }
    if (tid == 0) {
        offs[E] = total;
        n_active[layer] = total_active;
    }
    for (int i = total_active + tid; i < E; i += GROUP_THREADS) act[i] = -1;
    // ids outside [0, E)
    int bad = 0;
    for (int wc = tid; wc < nwc; wc += GROUP_THREADS) bad += h[(long long)wc * (E + 1) + E];
    int bad_total;
    (void)block_exclusive_scan(bad, &bad_total, buf);
    if (tid == 0) n_invalid[layer] = bad_total;
}

__global__ __launch_bounds__(GROUP_THREADS) void group_scatter_kernel(
    const int32_t* __restrict__ idx, int n, int E, int nbits, int nwc,
    const int32_t* __restrict__ base, const int32_t* __restrict__ offsets,
    int32_t* __restrict__ token_pos)
{
    __shared__ int32_t cursor[GROUP_WAVES][MAX_E];
    const int layer = blockIdx.y, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int wc = blockIdx.x * GROUP_WAVES + wave;
    const int32_t* offs = offsets + (long long)layer * (E + 1);
    if (wc < nwc) {
        const int32_t* b = base + ((long long)layer * nwc + wc) * (E + 1);
        for (int e = lane; e < E; e += 64) cursor[wave][e] = offs[e] + b[e];
    }
    const int total = offs[E];
    __syncthreads();
    const int32_t* src = idx + (long long)layer * n;
    int32_t* dst = token_pos + (long long)layer * n;
    const long long first = (long long)wc * WAVE_ITEMS;
    for (int i = 0; i < WAVE_ITEMS; i += 64) {
        const long long p = first + i + lane;
        int32_t e = -1;
        if (p < n) e = src[p];
        const bool valid = (e >= 0 && e < E);
        // lanes with the same expert id
        uint64_t same = __ballot(valid);
        for (int b = 0; b < nbits; ++b) {
            const bool bit = (e >> b) & 1;
            const uint64_t set = __ballot(valid && bit);
            same &= bit ? set : ~set;
        }
        // the highest lane of each group takes the group's slots from the wave's cursor (one LDS atomic
        // per distinct expert) and hands the old value to the others; only this wave touches cursor[wave]
        const int leader = valid ? 63 - __clzll((long long)same) : lane;
        int old = 0;
        if (valid && lane == leader) old = atomicAdd(&cursor[wave][e], __popcll(same));
        old = __shfl(old, leader, 64);
        if (valid) dst[old + __popcll(same & ((1ull << lane) - 1ull))] = (int32_t)p;
        // the unused tail of token_pos
        if (p < n && p >= total) dst[p] = -1;
    }
}


// ---------------------------------------------------------------------------
// P workgroups of WAVES waves per layer, everything in LDS.
//   sub            positions per (part, wave): the layer is cut into P parts of WAVES sub-spans
//   lhA[w][e]      (P > 1) wave w's count of expert e over its share [w*sub*P, (w+1)*sub*P) of the
//                  WHOLE layer: summed over w it gives counts, summed over the waves that lie before
//                  this workgroup's part it gives the selections of e that precede the part
//   lhB[w][e]      phase 1: count of e in this part's sub-span w; phase 2: turned into the wave's first
//                  slot for that expert in the part's local list; phase 3: the wave's cursor
//   gb[e]          global slot of local list entry i of expert e is gb[e] + i
//   list[i]        the part's selections grouped by expert, (expert << 16) | position
// Parts, sub-spans, batches and lanes are all visited in ascending position, so
// groups come out in ascending position as in the three-launch path.
// ---------------------------------------------------------------------------
static constexpr int FUSED_REGS = 32;                               // positions per lane and sub-span, kept in registers
static constexpr int FUSED_MAX_ITEMS = 16 * 64 * FUSED_REGS;        // 32768: positions must also fit 16 bits
static constexpr size_t FUSED_MAX_LDS = 160 * 1024 - 512;           // per workgroup on gfx950, less the static part

template <int WAVES>
__global__ __launch_bounds__(WAVES * 64) void group_fused_kernel(
    const int32_t* __restrict__ idx, int n, int E, int nbits, int P, int sub,
    int32_t* __restrict__ counts, int32_t* __restrict__ offsets, int32_t* __restrict__ token_pos,
    int32_t* __restrict__ active, int32_t* __restrict__ n_active, int32_t* __restrict__ n_invalid)
{
    constexpr int THREADS = WAVES * 64;
    extern __shared__ int32_t smem[];
    __shared__ int32_t wave_tot[WAVES][3];
    const int layer = blockIdx.y, part = blockIdx.x;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int EP = E + 1;
    const bool split = P > 1;
    int32_t* lhB = smem;                                   // [WAVES][EP]
    int32_t* lhA = smem + WAVES * EP;                      // [WAVES][EP], only when split
    int32_t* gb = lhA + (split ? WAVES * EP : 0);          // [E]
    int32_t* list = gb + E;                                // [sub * WAVES]
    const int32_t* src = idx + (long long)layer * n;
    int32_t* dst = token_pos + (long long)layer * n;
    for (int i = tid; i < (split ? 2 : 1) * WAVES * EP; i += THREADS) smem[i] = 0;
    __syncthreads();

    // whole layer, counted by wave shares (skipped when the workgroup owns the whole layer)
    if (split) {
        int32_t* mineA = lhA + wave * EP;
        const int spanA = sub * P, firstA = wave * spanA;
        constexpr int NB = 8;                               // loads in flight
#pragma unroll 1
        for (int j0 = 0; j0 < spanA; j0 += 64 * NB) {
            int32_t e8[NB];
            bool in8[NB];
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                const int p = firstA + j0 + 64 * u + lane;
                in8[u] = (j0 + 64 * u < spanA && p < n);
                e8[u] = in8[u] ? src[p] : 0;
            }
#pragma unroll
            for (int u = 0; u < NB; ++u)
                if (in8[u]) atomicAdd(&mineA[(e8[u] >= 0 && e8[u] < E) ? e8[u] : E], 1);
        }
        __builtin_amdgcn_sched_barrier(0);                 // keep the next phase's loads out of this loop's registers
    }
    // this part's sub-span of this wave, fetched once and kept in registers for both passes:
    // ev[j] = id at position first + 64*j + lane
    const int plen = sub * WAVES, pstart = part * plen;
    const int first = pstart + wave * sub;
    int32_t* mine = lhB + wave * EP;
    int32_t ev[FUSED_REGS];
#pragma unroll
    for (int j = 0; j < FUSED_REGS; ++j) {
        const int p = first + 64 * j + lane;
        ev[j] = (64 * j < sub && p < n) ? src[p] : -1;
    }
#pragma unroll
    for (int j = 0; j < FUSED_REGS; ++j) {
        const int p = first + 64 * j + lane;
        if (64 * j < sub && p < n) atomicAdd(&mine[(ev[j] >= 0 && ev[j] < E) ? ev[j] : E], 1);
    }
    __syncthreads();

    // per expert: sums over the waves -> count in the layer, count before this part, count in this part
    // with each wave's first slot.  Thread t owns expert t, so a scan over threads is a scan over experts.
    int cnt = 0, cnt_mine = 0, before = 0;
    const int e_own = tid;
    if (e_own < E) {
        int run = 0;
#pragma unroll 4
        for (int w = 0; w < WAVES; ++w) {
            const int c = lhB[w * EP + e_own];
            lhB[w * EP + e_own] = run;
            run += c;
        }
        cnt_mine = run;
        cnt = run;
        if (split) {
            cnt = 0;
            const int w0 = part * (WAVES / P);             // waves whose share lies before this part
#pragma unroll 4
            for (int w = 0; w < WAVES; ++w) {
                const int c = lhA[w * EP + e_own];
                if (w < w0) before += c;
                cnt += c;
            }
        }
    }
    // block-wide exclusive scans of cnt, cnt_mine and (cnt > 0): wave scan with shuffles, wave totals through LDS
    int incl = cnt, incl_m = cnt_mine, incl_a = (cnt > 0);
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int a = __shfl_up(incl, off, 64), m = __shfl_up(incl_m, off, 64), b = __shfl_up(incl_a, off, 64);
        if (lane >= off) { incl += a; incl_m += m; incl_a += b; }
    }
    if (lane == 63) { wave_tot[wave][0] = incl; wave_tot[wave][1] = incl_m; wave_tot[wave][2] = incl_a; }
    __syncthreads();
    int woff = 0, woff_m = 0, woff_a = 0, total = 0, total_m = 0, total_a = 0;
#pragma unroll 4
    for (int w = 0; w < WAVES; ++w) {
        const int a = wave_tot[w][0], m = wave_tot[w][1], b = wave_tot[w][2];
        if (w < wave) { woff += a; woff_m += m; woff_a += b; }
        total += a; total_m += m; total_a += b;
    }
    const int off_e = woff + incl - cnt, loc_e = woff_m + incl_m - cnt_mine, aoff = woff_a + incl_a - (cnt > 0);
    if (e_own < E) {
        gb[e_own] = off_e + before - loc_e;
#pragma unroll 4
        for (int w = 0; w < WAVES; ++w) lhB[w * EP + e_own] += loc_e;      // first local slot of wave w for this expert
    }
    if (part == 0) {                                        // every part knows the layer's totals; one writes them
        int32_t* offs = offsets + (long long)layer * EP;
        int32_t* act = active + (long long)layer * E;
        if (e_own < E) {
            counts[(long long)layer * E + e_own] = cnt;
            offs[e_own] = off_e;
            if (cnt > 0) act[aoff] = e_own;
        }
        for (int i = total_a + tid; i < E; i += THREADS) act[i] = -1;
        if (tid == 0) {
            offs[E] = total;
            n_active[layer] = total_a;
            int bad = 0;
            const int32_t* h = split ? lhA : lhB;
            for (int w = 0; w < WAVES; ++w) bad += h[w * EP + E];
            n_invalid[layer] = bad;
        }
    }
    __syncthreads();

    // scatter: lanes holding the same expert find each other with ballots over
    // the id bits; the highest such lane takes the group's slots from the
    // wave's cursor with one LDS atomic and hands the old value to the others.
    // The part's list is assembled in LDS (scattered 4-byte stores to global memory go
    // through the memory pipeline one address at a time) and written out in order.
#pragma unroll
    for (int j = 0; j < FUSED_REGS; ++j) {
        if (64 * j >= sub) break;                           // wave-uniform
        const int p = first + 64 * j + lane;
        const int32_t e = ev[j];
        const bool valid = (p < n && e >= 0 && e < E);
        uint64_t same = __ballot(valid);
        for (int b = 0; b < nbits; ++b) {
            const bool bit = (e >> b) & 1;
            const uint64_t set = __ballot(valid && bit);
            same &= bit ? set : ~set;
        }
        const int leader = valid ? 63 - __clzll((long long)same) : lane;
        int old = 0;
        if (valid && lane == leader) old = atomicAdd(&mine[e], __popcll(same));
        old = __shfl(old, leader, 64);
        if (valid) list[old + __popcll(same & ((1ull << lane) - 1ull))] = (e << 16) | p;
    }
    __syncthreads();
    for (int i = tid; i < total_m; i += THREADS) {
        const int32_t v = list[i];
        dst[gb[v >> 16] + i] = v & 0xFFFF;
    }
    // -1 fills the unused tail of the layer's list; each part fills its own stretch of it
    const int pend = (pstart + plen < n) ? pstart + plen : n;
    for (int i = (total > pstart ? total : pstart) + tid; i < pend; i += THREADS) dst[i] = -1;
}

// How a layer of n selections is run by the single-launch kernel: waves per workgroup, parts, positions per
// (part, wave), LDS bytes; ok = false when it does not fit (then the three-launch path serves the layer).
struct FusedPlan {
    bool ok;
    int waves, P, sub;
    size_t lds;
};
static FusedPlan fused_plan(long long n, int E)
{
    FusedPlan f{false, 16, 1, 64, 0};
    if (n > FUSED_MAX_ITEMS) return f;
    // short layers: a small workgroup (the per-expert loops over waves are what a short layer pays for)
    f.waves = (n <= 2048 && E <= 256) ? 4 : 16;
    // long layers with few enough experts for two histograms: up to 8 parts of at least ~2048 positions
    if (f.waves == 16 && E <= 256) {
        while (f.P < 8 && n > 2048ll * f.P * 2) f.P *= 2;
    }
    for (;; f.P /= 2) {
        const long long per = (long long)f.P * f.waves * 64;
        f.sub = (int)(((n + per - 1) / per) * 64);
        if (f.sub < 64) f.sub = 64;
        f.lds = sizeof(int32_t) * ((size_t)(f.P > 1 ? 2 : 1) * f.waves * (size_t)(E + 1) + (size_t)E +
                                   (size_t)f.sub * f.waves);
        if (f.sub <= 64 * FUSED_REGS && f.lds <= FUSED_MAX_LDS) { f.ok = true; return f; }
        if (f.P == 1) return f;
    }
}

// the single-launch kernel serves the layer (no workspace)
static bool fused_fits(long long n, int E) { return fused_plan(n, E).ok; }

size_t group_workspace_bytes(int L, int T, int k, int E)
{
    const long long n = (long long)T * k;
    if (fused_fits(n, E)) return 0;
    return sizeof(int32_t) * (size_t)L * (size_t)wave_chunks(n) * (size_t)(E + 1);
}

hipError_t launch_group(const int32_t* idx, int L, int T, int k, int E,
                        int32_t* counts, int32_t* offsets, int32_t* token_pos,
                        int32_t* active, int32_t* n_active, int32_t* n_invalid,
                        void* workspace, hipStream_t stream)
{
    const int n = T * k;
    const int nwc = wave_chunks(n);
    const int nbc = block_chunks(n);
    int nbits = 0;
    while ((1 << nbits) < E) ++nbits;
    const FusedPlan f = fused_plan(n, E);
    if (f.ok) {
        hipError_t err;
        if (f.waves == 4) {
            static LdsLimit limit;
            err = ensure_lds_limit(limit, (const void*)group_fused_kernel<4>, f.lds);
            if (err != hipSuccess) return err;
            hipLaunchKernelGGL(group_fused_kernel<4>, dim3(f.P, L), dim3(256), f.lds, stream, idx, n, E, nbits, f.P,
                               f.sub, counts, offsets, token_pos, active, n_active, n_invalid);
        } else {
            static LdsLimit limit;
            err = ensure_lds_limit(limit, (const void*)group_fused_kernel<16>, f.lds);
            if (err != hipSuccess) return err;
            hipLaunchKernelGGL(group_fused_kernel<16>, dim3(f.P, L), dim3(1024), f.lds, stream, idx, n, E, nbits,
                               f.P, f.sub, counts, offsets, token_pos, active, n_active, n_invalid);
        }
        return hipGetLastError();
    }
    int32_t* hist = (int32_t*)workspace;
    if (nbc > 0)
        hipLaunchKernelGGL(group_hist_kernel, dim3(nbc, L), dim3(GROUP_THREADS), 0, stream, idx, n, E, nwc, hist);
    hipLaunchKernelGGL(group_scan_kernel, dim3(L), dim3(GROUP_THREADS), 0, stream, E, nwc, hist, counts,
                       offsets, active, n_active, n_invalid);
    if (nbc > 0)
        hipLaunchKernelGGL(group_scatter_kernel, dim3(nbc, L), dim3(GROUP_THREADS), 0, stream, idx, n, E,
                           nbits, nwc, hist, offsets, token_pos);
    return hipGetLastError();
}

}  // namespace paep

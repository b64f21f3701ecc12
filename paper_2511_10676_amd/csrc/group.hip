// Per-expert grouping of the selected expert ids: histogram, exclusive scan,
// stable index compaction (a counting sort by expert id).  This produces the
// prefetch list that the paper's workflow (section 4.2, third stage) derives
// from the selection: which experts are needed and which tokens need each of
// them.
//
// A layer is cut into P parts, one workgroup each (group_fused_kernel); a part
// assembles its selections grouped by expert in LDS and writes them out as
// runs, one per expert, behind the selections of that expert in earlier
// parts.  For that a workgroup has to know two numbers per expert: how many
// selections the whole layer has (the layer's offsets) and how many lie before
// its own part.  Where they come from depends on the layer's length:
//   up to FUSED_MAX_ITEMS selections   one launch: the workgroups of a layer do
//            not talk to each other, every one of them counts the WHOLE layer
//            (counting is the cheap phase, one LDS atomic per selection).  No
//            workspace, no second launch, no waiting.
//   longer   a first launch counts every part once (group_part_hist_kernel)
//            into the workspace, hist[layer][part][E + 1] (slot E counts ids
//            outside [0, E)); the workgroups of the second launch sum the
//            columns of that matrix themselves.  With more than SCAN_PARTS
//            parts a launch in between turns the columns into running sums
//            (group_scan_parts_kernel), so that the column sums stay linear in
//            the layer's length.
// Order inside a group is ascending position because parts, waves, batches
// and lanes are all visited in ascending order.
#include "paep_internal.h"

namespace paep {

static constexpr int PART_WAVES = 16;                   // waves per workgroup on layers that take the workspace
static constexpr int PART_SUB = 512;                    // positions per wave of a part (doubled while parts > SCAN_PARTS)
static constexpr int SCAN_PARTS = 64;                   // more parts than this: columns are scanned by a launch of their own

// counts of one part: hist[layer][part][0..E], 1024 threads, grid (P, L)
__global__ __launch_bounds__(PART_WAVES * 64) void group_part_hist_kernel(
    const int32_t* __restrict__ idx, int n, int E, int P, int plen, int32_t* __restrict__ hist)
{
    constexpr int THREADS = PART_WAVES * 64;
    extern __shared__ int32_t smem[];                   // [E + 1]
    const int layer = blockIdx.y, part = blockIdx.x, tid = threadIdx.x;
    for (int e = tid; e <= E; e += THREADS) smem[e] = 0;
    __syncthreads();
    const int32_t* src = idx + (long long)layer * n;
    const int pstart = part * plen;
    constexpr int NB = 8;                               // loads in flight
#pragma unroll 1
    for (int j0 = 0; j0 < plen; j0 += THREADS * NB) {
        int32_t e8[NB];
        bool in8[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const int j = j0 + THREADS * u + tid;
            in8[u] = (j < plen && pstart + j < n);
            e8[u] = in8[u] ? src[pstart + j] : 0;
        }
#pragma unroll
        for (int u = 0; u < NB; ++u)
            if (in8[u]) atomicAdd(&smem[(e8[u] >= 0 && e8[u] < E) ? e8[u] : E], 1);
    }
    __syncthreads();
    int32_t* dst = hist + ((long long)layer * (P + 1) + part) * (E + 1);
    for (int e = tid; e <= E; e += THREADS) dst[e] = smem[e];
}

// hist[layer][q][e] -> selections of e in parts before q; row P receives the column totals.  Grid (L).
__global__ __launch_bounds__(256) void group_scan_parts_kernel(int E, int P, int32_t* __restrict__ hist)
{
    int32_t* h = hist + (long long)blockIdx.x * (P + 1) * (E + 1);
    for (int e = threadIdx.x; e <= E; e += 256) {
        int run = 0;
        for (int q0 = 0; q0 < P; q0 += 16) {            // 16 loads in flight, then their running sums
            int c[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) c[u] = (q0 + u < P) ? h[(long long)(q0 + u) * (E + 1) + e] : 0;
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                if (q0 + u < P) h[(long long)(q0 + u) * (E + 1) + e] = run;
                run += c[u];
            }
        }
        h[(long long)P * (E + 1) + e] = run;
    }
}


// ---------------------------------------------------------------------------
// P workgroups of WAVES waves per layer, everything in LDS.
//   sub            positions per (part, wave): the layer is cut into P parts of WAVES sub-spans
//   lhA[w][e]      (P > 1, no workspace) wave w's count of expert e over its share [w*sub*P, (w+1)*sub*P)
//                  of the WHOLE layer: summed over w it gives counts, summed over the waves that lie
//                  before this workgroup's part it gives the selections of e that precede the part
//   part_hist      (PRE) the parts' counts from group_part_hist_kernel instead, hist[layer][q][e]; with
//                  `scanned` row q already holds the sum of the rows before it and row P the totals
//   lhB[w][e]      phase 1: count of e in this part's sub-span w; phase 2: turned into the wave's first
//                  slot for that expert in the part's local list; phase 3: the wave's cursor
//   gb[e]          global slot of local list entry i of expert e is gb[e] + i
//   list[i]        the part's selections grouped by expert, (expert << 16) | position inside the part
// ---------------------------------------------------------------------------
static constexpr int FUSED_REGS = 32;                               // most positions per lane and sub-span (kept in registers)
static constexpr int FUSED_MAX_ITEMS = 16 * 64 * FUSED_REGS;        // 32768 per part: positions must also fit 16 bits
static constexpr int COLSUM_INTS = 1028;                            // partial column sums: at most max(1024, E + 1) of them
static constexpr size_t FUSED_MAX_LDS = 160 * 1024 - 512 - 8 * COLSUM_INTS;   // per workgroup on gfx950, less the static part

// The lanes of the wave that hold the same id as this one (valid lanes only; ids below 2^nbits2, nbits2 even).
// Per id bit: one ballot, and every lane keeps the lanes whose bit equals its own.
__device__ __forceinline__ uint64_t lanes_with_same_id(int32_t e, bool valid, int nbits2)
{
    uint64_t same = __ballot(valid);
    uint32_t lo = (uint32_t)same, hi = (uint32_t)(same >> 32);
#pragma unroll 1
    for (int b = 0; b < nbits2; b += 2) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int32_t mine = __builtin_amdgcn_sbfe(e, b + u, 1);          // 0 or -1: this lane's bit, spread
            const uint64_t set = __ballot(mine != 0);
            lo &= ~((uint32_t)set ^ (uint32_t)mine);
            hi &= ~((uint32_t)(set >> 32) ^ (uint32_t)mine);
        }
    }
    return ((uint64_t)hi << 32) | lo;
}

template <int WAVES, bool PRE, int REGS>
__global__ __launch_bounds__(WAVES * 64, (WAVES == 16 && REGS <= 8) ? 8 : WAVES / 4) void group_fused_kernel(
    const int32_t* __restrict__ idx, int n, int E, int nbits, int P, int sub,
    const int32_t* __restrict__ part_hist, int scanned, int32_t* __restrict__ counts, int32_t* __restrict__ offsets, int32_t* __restrict__ token_pos,
    int32_t* __restrict__ active, int32_t* __restrict__ n_active, int32_t* __restrict__ n_invalid)
{
    constexpr int THREADS = WAVES * 64;
    extern __shared__ int32_t smem[];
    __shared__ int32_t wave_tot[WAVES][3];
    __shared__ int32_t colsum[PRE ? 2 * COLSUM_INTS : 1];
    const int layer = blockIdx.y, part = blockIdx.x;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int EP = E + 1;
    const bool split = !PRE && P > 1;
    int32_t* lhB = smem;                                   // [WAVES][EP]
    int32_t* lhA = smem + WAVES * EP;                      // [WAVES][EP], only when counting the layer here
    int32_t* gb = lhA + (split ? WAVES * EP : 0);          // [E]
    int32_t* list = gb + E;                                // [sub * WAVES]
    const int32_t* src = idx + (long long)layer * n;
    int32_t* dst = token_pos + (long long)layer * n;

    // whole layer, counted by wave shares (skipped when the workgroup owns the whole layer or has the parts' counts)
    if (split) {
        for (int i = tid; i < 2 * WAVES * EP; i += THREADS) smem[i] = 0;
        __syncthreads();
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
    int32_t ev[REGS];
#pragma unroll
    for (int j = 0; j < REGS; ++j) {
        const int p = first + 64 * j + lane;
        ev[j] = (64 * j < sub && p < n) ? src[p] : -1;
    }
    // the parts' counts (PRE), summed by columns while the ids arrive: thread (r, e) takes the rows r, r + R, ...
    // of column e (column E: the ids outside [0, E)); the R partial sums of a column meet in LDS.  Rows already
    // turned into running sums need no adding up: row `part` and the totals' row are copied.
    int col_groups = 1;
    if (PRE) {
        const int32_t* ph = part_hist + (long long)layer * (P + 1) * EP;
        if (scanned) {
            for (int e = tid; e < EP; e += THREADS) {
                colsum[e] = ph[(long long)P * EP + e];
                colsum[EP + e] = ph[(long long)part * EP + e];
            }
        } else {
            col_groups = THREADS > EP ? THREADS / EP : 1;
            for (int it = tid; it < col_groups * EP; it += THREADS) {
                const int r = it / EP, e = it - r * EP;
                int all = 0, bef = 0;
#pragma unroll 8
                for (int q = r; q < P; q += col_groups) {
                    const int c = ph[(long long)q * EP + e];
                    if (q < part) bef += c;
                    all += c;
                }
                colsum[r * EP + e] = all;
                colsum[(col_groups + r) * EP + e] = bef;
            }
        }
    }
    if (!split) {                                           // histograms cleared while the loads are under way
        for (int i = tid; i < WAVES * EP; i += THREADS) smem[i] = 0;
        __syncthreads();
    }
#pragma unroll
    for (int j = 0; j < REGS; ++j) {
        const int p = first + 64 * j + lane;
        const bool good = (uint32_t)ev[j] < (uint32_t)E;
        if (64 * j < sub && p < n) atomicAdd(&mine[good ? ev[j] : E], 1);
        if (!good) ev[j] = -1;                              // from here on: an expert id, or -1 for nothing to place
    }
    __syncthreads();

    // per expert: sums over the waves -> count in the layer, count before this part, count in this part
    // with each wave's first slot.  Thread t owns expert t, so a scan over threads is a scan over experts.
    int cnt = 0, cnt_mine = 0, before = 0;
    const int e_own = tid;
    int first_slot[WAVES];                                  // of wave w for this expert, relative to the expert's run
    if (e_own < E) {
        int run = 0;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            first_slot[w] = run;
            run += lhB[w * EP + e_own];
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
        if (PRE) {
            cnt = before = 0;
            for (int r = 0; r < col_groups; ++r) {
                cnt += colsum[r * EP + e_own];
                before += colsum[(col_groups + r) * EP + e_own];
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
#pragma unroll
        for (int w = 0; w < WAVES; ++w) lhB[w * EP + e_own] = first_slot[w] + loc_e;   // wave w's cursor for this expert
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
            if (PRE) {
                for (int r = 0; r < col_groups; ++r) bad += colsum[r * EP + E];
            } else {
                const int32_t* h = split ? lhA : lhB;
                for (int w = 0; w < WAVES; ++w) bad += h[w * EP + E];
            }
            n_invalid[layer] = bad;
        }
    }
    __syncthreads();

    // scatter: lanes holding the same expert find each other with ballots over the id bits; all of them read
    // the wave's cursor for that expert, the lowest of them moves it on (only this wave touches its cursors, and
    // its LDS accesses are carried out in program order).  The part's list is assembled in LDS (scattered
    // 4-byte stores to global memory go through the memory pipeline one address at a time) and written out in
    // order.
    const uint64_t below = (1ull << lane) - 1ull;
    const int nbits2 = (nbits + 1) & ~1;
#pragma unroll
    for (int j = 0; j < REGS; ++j) {
        if (64 * j >= sub) break;                           // wave-uniform
        const int32_t e = ev[j];
        const bool valid = e >= 0;
        const uint64_t same = lanes_with_same_id(e, valid, nbits2);
        const int rank = __popcll(same & below);
        if (valid) {
            const int old = mine[e];
            if (rank == 0) mine[e] = old + __popcll(same);
            list[old + rank] = (e << 16) | (wave * sub + 64 * j + lane);
        }
    }
    __syncthreads();
    for (int i = tid; i < total_m; i += THREADS) {
        const int32_t v = list[i];
        dst[gb[v >> 16] + i] = pstart + (v & 0xFFFF);
    }
    // -1 fills the unused tail of the layer's list; each part fills its own stretch of it
    const int pend = (pstart + plen < n) ? pstart + plen : n;
    for (int i = (total > pstart ? total : pstart) + tid; i < pend; i += THREADS) dst[i] = -1;
}

// How a layer of n selections is run: waves per workgroup, parts, positions per (part, wave), LDS bytes of
// the grouping kernel; pre = the parts are counted by a launch of their own (workspace), scan = and their
// columns scanned by another.
struct FusedPlan {
    bool pre, scan;
    int waves, P, sub;
    size_t lds;
};
static size_t fused_lds(int hists, int waves, int E, int sub)
{
    return sizeof(int32_t) * ((size_t)hists * waves * (size_t)(E + 1) + (size_t)E + (size_t)sub * waves);
}
static FusedPlan fused_plan(long long n, int E)
{
    FusedPlan f{false, false, 16, 1, 64, 0};
    if (n <= FUSED_MAX_ITEMS) {
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
            f.lds = fused_lds(f.P > 1 ? 2 : 1, f.waves, E, f.sub);
            if (f.sub <= 64 * FUSED_REGS && f.lds <= FUSED_MAX_LDS) return f;
            if (f.P == 1) break;
        }
    }
    // parts of PART_SUB positions per wave; longer ones (as far as LDS allows) while there would be more than
    // SCAN_PARTS of them
    f.pre = true;
    f.waves = PART_WAVES;
    f.sub = PART_SUB;
    while (f.sub > 64 && fused_lds(1, f.waves, E, f.sub) > FUSED_MAX_LDS) f.sub /= 2;
    for (;;) {
        const long long plen = (long long)f.sub * f.waves;
        f.P = (int)((n + plen - 1) / plen);
        if (f.P <= SCAN_PARTS || f.sub * 2 > 64 * FUSED_REGS || fused_lds(1, f.waves, E, f.sub * 2) > FUSED_MAX_LDS)
            break;
        f.sub *= 2;
    }
    f.scan = f.P > SCAN_PARTS;
    f.lds = fused_lds(1, f.waves, E, f.sub);
    return f;
}

size_t group_workspace_bytes(int L, int T, int k, int E)
{
    const long long n = (long long)T * k;
    const FusedPlan f = fused_plan(n, E);
    if (!f.pre) return 0;
    return sizeof(int32_t) * (size_t)L * (size_t)(f.P + 1) * (size_t)(E + 1);
}

template <int WAVES, bool PRE, int REGS>
static hipError_t launch_fused_regs(const FusedPlan& f, const int32_t* idx, int L, int n, int E, int nbits,
                               const int32_t* hist, int32_t* counts, int32_t* offsets, int32_t* token_pos,
                               int32_t* active, int32_t* n_active, int32_t* n_invalid, hipStream_t stream)
{
    static LdsLimit limit;
    const hipError_t err = ensure_lds_limit(limit, (const void*)group_fused_kernel<WAVES, PRE, REGS>, f.lds);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL((group_fused_kernel<WAVES, PRE, REGS>), dim3(f.P, L), dim3(WAVES * 64), f.lds, stream, idx, n, E,
                       nbits, f.P, f.sub, hist, f.scan ? 1 : 0, counts, offsets, token_pos, active, n_active,
                       n_invalid);
    return hipGetLastError();
}

// compiled for 8 positions per lane (short sub-spans: two workgroups of 16 waves share a compute unit) and for 32
template <int WAVES, bool PRE>
static hipError_t launch_fused(const FusedPlan& f, const int32_t* idx, int L, int n, int E, int nbits,
                               const int32_t* hist, int32_t* counts, int32_t* offsets, int32_t* token_pos,
                               int32_t* active, int32_t* n_active, int32_t* n_invalid, hipStream_t stream)
{
    if (f.sub <= 64 * 8)
        return launch_fused_regs<WAVES, PRE, 8>(f, idx, L, n, E, nbits, hist, counts, offsets, token_pos, active,
                                                n_active, n_invalid, stream);
    if constexpr (WAVES == 16)
        return launch_fused_regs<WAVES, PRE, FUSED_REGS>(f, idx, L, n, E, nbits, hist, counts, offsets, token_pos,
                                                         active, n_active, n_invalid, stream);
    return hipErrorInvalidValue;                            // the plan gives 4-wave workgroups short sub-spans only
}

hipError_t launch_group(const int32_t* idx, int L, int T, int k, int E,
                        int32_t* counts, int32_t* offsets, int32_t* token_pos,
                        int32_t* active, int32_t* n_active, int32_t* n_invalid,
                        void* workspace, hipStream_t stream)
{
    const int n = T * k;
    int nbits = 0;
    while ((1 << nbits) < E) ++nbits;
    const FusedPlan f = fused_plan(n, E);
    if (!f.pre) {
        if (f.waves == 4)
            return launch_fused<4, false>(f, idx, L, n, E, nbits, nullptr, counts, offsets, token_pos, active,
                                          n_active, n_invalid, stream);
        return launch_fused<16, false>(f, idx, L, n, E, nbits, nullptr, counts, offsets, token_pos, active,
                                       n_active, n_invalid, stream);
    }
    int32_t* hist = (int32_t*)workspace;
    hipLaunchKernelGGL(group_part_hist_kernel, dim3(f.P, L), dim3(PART_WAVES * 64), sizeof(int32_t) * (E + 1),
                       stream, idx, n, E, f.P, f.sub * f.waves, hist);
    if (f.scan) hipLaunchKernelGGL(group_scan_parts_kernel, dim3(L), dim3(256), 0, stream, E, f.P, hist);
    return launch_fused<PART_WAVES, true>(f, idx, L, n, E, nbits, hist, counts, offsets, token_pos, active,
                                          n_active, n_invalid, stream);
}

}  // namespace paep

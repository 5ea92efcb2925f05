// Per-lookup planning pass (paper: step a, "Setting Computation Mask" /
// "Implicit Computation Mask"): decide which blocks of the volume are computed.
//
// The paper groups source pixels by 8x8 source tile and lets each tile vote
// for the target blocks it needs.  Here the grouping is by *target*: at level l
// the integer origin of a query's (2r+2)^2 footprint, o = floor(c / 2^l) - r,
// falls in a cell of side b_l = 8 >> l, and all queries of one cell share the
// fixed window of (b_l + 2r + 1)^2 target pixels that starts at the cell's
// corner.  A work item is (cell, group of <= 64 of its queries); the blocks of
// the volume that get computed are exactly those items' window x group
// products.  Queries whose footprint misses the level entirely are written as
// zeros here and never reach the contraction.
//
// Three kernels: count (cell id + slot per query-level), scan (cell offsets,
// per-level item lists, statistics), scatter (queries sorted by cell).
#include "corr_internal.h"

namespace {

struct BinArgs {
    const float* coords;   // [B][2][H*W]
    float* out;            // [B][L*K*K][H*W]
    int B, HW, W, L, r;
    LevelGeom lv[CORR_MAX_L];
    int* bin_count;
    int* q_bin;
    int* q_rank;
};

__global__ __launch_bounds__(256) void bin_count_kernel(BinArgs a) {
    const int q = blockIdx.x * blockDim.x + threadIdx.x;   // b*HW + pixel
    const int BN = a.B * a.HW;
    const bool real = q < BN;                 // lanes past the end stay for the shuffles
    const int b = real ? q / a.HW : 0, p = real ? q - b * a.HW : 0;
    const float cx = real ? a.coords[((size_t)b * 2 + 0) * a.HW + p] : NAN;
    const float cy = real ? a.coords[((size_t)b * 2 + 1) * a.HW + p] : NAN;
    const int K = 2 * a.r + 1;
    // comparisons are false for NaN, so non-finite coordinates are "not ok"
    const bool finite_ok = (fabsf(cx) <= CORR_COORD_LIMIT) && (fabsf(cy) <= CORR_COORD_LIMIT);
    for (int l = 0; l < a.L; ++l) {
        const LevelGeom g = a.lv[l];
        const float inv = __uint_as_float((uint32_t)(127 - l) << 23);   // 2^-l, exact
        int bin = -1;
        if (finite_ok) {
            const int ox = (int)floorf(cx * inv) - a.r;
            const int oy = (int)floorf(cy * inv) - a.r;
            // the footprint ox..ox+K touches the level iff ox+K >= 0 and ox <= W-1
            if (ox + K >= 0 && ox <= g.W - 1 && oy + K >= 0 && oy <= g.H - 1) {
                const int bx = (ox + CORR_PAD) >> g.shift;
                const int by = (oy + CORR_PAD) >> g.shift;
                bin = g.bin_base + (b * g.nby + by) * g.nbx + bx;
            }
        }
        // Neighbouring pixels mostly fall in the same cell: one atomic per run of
        // equal cell ids among consecutive lanes, the rest of the run takes offsets.
        const int lane = threadIdx.x & 63;
        const int prev = __shfl_up(bin, 1, 64);
        const bool head = (lane == 0) || (bin != prev);
        const unsigned long long heads = __ballot(head);
        const unsigned long long upto = (lane == 63) ? ~0ull : ((2ull << lane) - 1ull);
        const int head_lane = 63 - __clzll((long long)(heads & upto));
        const unsigned long long above = heads & ~upto;
        const int next = above ? (__ffsll((long long)above) - 1) : 64;
        int base = 0;
        if (head && bin >= 0) base = atomicAdd(&a.bin_count[bin], next - lane);
        const int rank = __shfl(base, head_lane, 64) + (lane - head_lane);
        if (bin < 0 && real) {
            float* o = a.out + ((size_t)b * a.L * K * K + (size_t)l * K * K) * a.HW + p;
            for (int t = 0; t < K * K; ++t) o[(size_t)t * a.HW] = 0.0f;
        }
        if (real) {
            a.q_bin[(size_t)l * BN + q] = bin;
            a.q_rank[(size_t)l * BN + q] = rank;
        }
    }
}

struct ScanArgs {
    int nbins, L, BN;
    int level_end[CORR_MAX_L];       // bin_base of the next level
    int win_pts[CORR_MAX_L];         // window points per level
    int* bin_count;
    int* bin_off;
    int4* items;
    int* level_item_off;
    long long* stats;
};

// Single workgroup: exclusive scan of the counts (query offsets) and of the
// per-cell item counts, in tiles of 4096 cells (one int4 per thread, coalesced);
// writes the item list in cell order, hence level-major.
__global__ __launch_bounds__(1024) void bin_scan_kernel(ScanArgs a) {
    __shared__ int s_wc[16], s_wi[16];
    __shared__ unsigned long long s_stats[CORR_NSTATS];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    if (t < CORR_NSTATS) s_stats[t] = 0;
    int carry_c = 0, carry_i = 0;
    long long mma = 0, used = 0, nit = 0, nq = 0;
    int cur = -1;
    auto flush = [&]() {
        if (cur >= 0 && (nit | nq)) {
            atomicAdd(&s_stats[8 + 4 * cur + 0], (unsigned long long)nit);
            atomicAdd(&s_stats[8 + 4 * cur + 1], (unsigned long long)mma);
            atomicAdd(&s_stats[8 + 4 * cur + 2], (unsigned long long)used);
            atomicAdd(&s_stats[8 + 4 * cur + 3], (unsigned long long)nq);
        }
        mma = used = nit = nq = 0;
    };
    const int ntiles = (a.nbins + 4095) / 4096;
    auto load_tile = [&](int tile) {
        const int g0 = tile * 4096 + t * 4;
        int4 c = make_int4(0, 0, 0, 0);
        if (g0 + 3 < a.nbins) c = *reinterpret_cast<const int4*>(a.bin_count + g0);
        else {
            if (g0 < a.nbins) c.x = a.bin_count[g0];
            if (g0 + 1 < a.nbins) c.y = a.bin_count[g0 + 1];
            if (g0 + 2 < a.nbins) c.z = a.bin_count[g0 + 2];
        }
        return c;
    };
    int4 nxt = load_tile(0);
    for (int tile = 0; tile < ntiles; ++tile) {
        const int4 c4 = nxt;
        if (tile + 1 < ntiles) nxt = load_tile(tile + 1);
        const int c[4] = {c4.x, c4.y, c4.z, c4.w};
        int csum = 0, isum = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) { csum += c[k]; isum += (c[k] + CORR_GROUP - 1) / CORR_GROUP; }
        int ci = csum, ii = isum;                   // inclusive scan within the wave
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int vc = __shfl_up(ci, d, 64), vi = __shfl_up(ii, d, 64);
            if (lane >= d) { ci += vc; ii += vi; }
        }
        __syncthreads();                            // previous tile's s_wc/s_wi fully consumed
        if (lane == 63) { s_wc[wave] = ci; s_wi[wave] = ii; }
        __syncthreads();
        int wc = 0, wi = 0, tot_c = 0, tot_i = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const int vc = s_wc[w], vi = s_wi[w];
            if (w < wave) { wc += vc; wi += vi; }
            tot_c += vc; tot_i += vi;
        }
        int coff = carry_c + wc + ci - csum, ioff = carry_i + wi + ii - isum;
        carry_c += tot_c; carry_i += tot_i;
        const int g0 = tile * 4096 + t * 4;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int g = g0 + k;
            if (g >= a.nbins) break;
            int level = 0;
            while (level < a.L - 1 && g >= a.level_end[level]) ++level;
            if (level != cur) { flush(); cur = level; }
            nq += c[k];
            // first cell of a level records where that level's items start
            if (g == (level == 0 ? 0 : a.level_end[level - 1])) a.level_item_off[level] = ioff;
            a.bin_off[g] = coff;
            a.bin_count[g] = 0;                     // ready for the next lookup
            for (int s = 0; s < c[k]; s += CORR_GROUP) {
                const int n = min(CORR_GROUP, c[k] - s);
                a.items[ioff++] = make_int4(g, coff + s, n, level);
                ++nit;
                mma += (long long)a.win_pts[level] * ((n + 15) & ~15);
                used += (long long)a.win_pts[level] * n;
            }
            coff += c[k];
        }
    }
    flush();
    __syncthreads();
    if (t == 0) {
        a.level_item_off[a.L] = carry_i;
        long long mma_all = 0, used_all = 0;
        for (int l = 0; l < CORR_MAX_L; ++l) { mma_all += s_stats[8 + 4 * l + 1]; used_all += s_stats[8 + 4 * l + 2]; }
        a.stats[0] = carry_i;                                   // items
        a.stats[1] = (long long)a.BN * a.L;                     // query-levels
        a.stats[2] = (long long)a.BN * a.L - carry_c;           // null query-levels
        a.stats[3] = mma_all;
        a.stats[4] = used_all;
    }
    if (t >= 8 && t < CORR_NSTATS) a.stats[t] = (long long)s_stats[t];
}

__global__ __launch_bounds__(256) void bin_scatter_kernel(const int* __restrict__ q_bin,
                                                          const int* __restrict__ q_rank,
                                                          const int* __restrict__ bin_off,
                                                          int* __restrict__ perm, int BN, int L) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= BN * L) return;
    const int bin = q_bin[i];
    if (bin >= 0) perm[bin_off[bin] + q_rank[i]] = i % BN;
}

}  // namespace

hipError_t launch_binning(corr_pyramid* p, const float* coords, int r, float* out, hipStream_t s) {
    const int HW = p->H * p->W, BN = p->B * HW;
    BinArgs a;
    a.coords = coords; a.out = out; a.B = p->B; a.HW = HW; a.W = p->W; a.L = p->L; a.r = r;
    for (int l = 0; l < CORR_MAX_L; ++l) a.lv[l] = p->lv[l];
    a.bin_count = p->bin_count; a.q_bin = p->q_bin; a.q_rank = p->q_rank;
    hipLaunchKernelGGL(bin_count_kernel, dim3((BN + 255) / 256), dim3(256), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    ScanArgs sc;
    sc.nbins = p->nbins; sc.L = p->L; sc.BN = BN;
    for (int l = 0; l < CORR_MAX_L; ++l) {
        sc.level_end[l] = (l + 1 < p->L) ? p->lv[l + 1].bin_base : p->nbins;
        const int ws = (1 << p->lv[l].shift) + 2 * r + 1;
        sc.win_pts[l] = ws * ws;
    }
    sc.bin_count = p->bin_count; sc.bin_off = p->bin_off; sc.items = p->items;
    sc.level_item_off = p->level_item_off; sc.stats = p->stats;
    hipLaunchKernelGGL(bin_scan_kernel, dim3(1), dim3(1024), 0, s, sc);
    e = hipGetLastError();
    if (e != hipSuccess) return e;

    hipLaunchKernelGGL(bin_scatter_kernel, dim3((BN * p->L + 255) / 256), dim3(256), 0, s,
                       p->q_bin, p->q_rank, p->bin_off, p->perm, BN, p->L);
    return hipGetLastError();
}

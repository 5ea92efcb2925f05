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
    if (q >= BN) return;
    const int b = q / a.HW, p = q - b * a.HW;
    const float cx = a.coords[((size_t)b * 2 + 0) * a.HW + p];
    const float cy = a.coords[((size_t)b * 2 + 1) * a.HW + p];
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
        int rank = 0;
        if (bin >= 0) {
            rank = atomicAdd(&a.bin_count[bin], 1);
        } else {
            float* o = a.out + ((size_t)b * a.L * K * K + (size_t)l * K * K) * a.HW + p;
            for (int t = 0; t < K * K; ++t) o[(size_t)t * a.HW] = 0.0f;
        }
        a.q_bin[(size_t)l * BN + q] = bin;
        a.q_rank[(size_t)l * BN + q] = rank;
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
// per-cell item counts; writes the item list in cell order, hence level-major.
__global__ __launch_bounds__(1024) void bin_scan_kernel(ScanArgs a) {
    __shared__ int s_cnt[1024], s_itm[1024];
    __shared__ long long s_red[1024];
    const int t = threadIdx.x;
    const int per = (a.nbins + 1023) / 1024;
    const int lo = t * per, hi = min(lo + per, a.nbins);
    int csum = 0, isum = 0;
    for (int g = lo; g < hi; ++g) {
        const int c = a.bin_count[g];
        csum += c;
        isum += (c + CORR_GROUP - 1) / CORR_GROUP;
    }
    s_cnt[t] = csum; s_itm[t] = isum;
    __syncthreads();
    // Hillis-Steele inclusive scan over 1024 partials
    for (int d = 1; d < 1024; d <<= 1) {
        int vc = 0, vi = 0;
        if (t >= d) { vc = s_cnt[t - d]; vi = s_itm[t - d]; }
        __syncthreads();
        s_cnt[t] += vc; s_itm[t] += vi;
        __syncthreads();
    }
    int coff = s_cnt[t] - csum, ioff = s_itm[t] - isum;
    long long mma = 0, used = 0;
    for (int g = lo; g < hi; ++g) {
        const int c = a.bin_count[g];
        int level = 0;
        while (level < a.L - 1 && g >= a.level_end[level]) ++level;
        // first cell of a level records where that level's items start
        if (g == (level == 0 ? 0 : a.level_end[level - 1])) a.level_item_off[level] = ioff;
        a.bin_off[g] = coff;
        a.bin_count[g] = 0;                       // ready for the next lookup
        for (int s = 0; s < c; s += CORR_GROUP) {
            const int n = min(CORR_GROUP, c - s);
            a.items[ioff++] = make_int4(g, coff + s, n, level);
            mma += (long long)a.win_pts[level] * ((n + 15) & ~15);
            used += (long long)a.win_pts[level] * n;
        }
        coff += c;
    }
    s_red[t] = mma;
    __syncthreads();
    for (int d = 512; d > 0; d >>= 1) { if (t < d) s_red[t] += s_red[t + d]; __syncthreads(); }
    const long long mma_all = s_red[0];
    __syncthreads();
    s_red[t] = used;
    __syncthreads();
    for (int d = 512; d > 0; d >>= 1) { if (t < d) s_red[t] += s_red[t + d]; __syncthreads(); }
    if (t == 1023) {
        a.level_item_off[a.L] = s_itm[1023];
        a.stats[0] = s_itm[1023];                               // items
        a.stats[1] = (long long)a.BN * a.L;                     // query-levels
        a.stats[2] = (long long)a.BN * a.L - s_cnt[1023];       // null query-levels
        a.stats[3] = mma_all;
        a.stats[4] = s_red[0];
    }
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

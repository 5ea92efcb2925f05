// Per-lookup planning pass (paper: step a, "Setting Computation Mask" /
// "Implicit Computation Mask"): decide which blocks of the volume are computed.
//
// The paper groups source pixels by 8x8 source tile and lets each tile vote
// for the target blocks it needs.  Here the grouping is by *target*: a query
// belongs to the cell (floor(cx) >> 3, floor(cy) >> 3) of its level-0 target.
// Since floor(c / 2^l) == floor(c) >> l, the footprint origins of a cell's
// queries lie, at level l, in one aligned run of max(8 >> l, 1) pixels per
// axis, so the cell owns one fixed window of (max(8 >> l, 1) + 2r + 1)^2
// target pixels per level.  A work item is (cell, group of <= 64 of its
// queries); the blocks of the volume that get computed are exactly the items'
// window x group products, for every level.  Queries out of range at every
// level are written as zeros here and never reach the contraction.
//
// Three kernels: count (cell id + slot per query), scan (cell offsets, item
// list, statistics), scatter (queries sorted by cell).
#include "corr_internal.h"

namespace {

struct BinArgs {
    const float* coords;   // [B][2][H*W]
    float* out;            // [B][L*K*K][H*W]
    int B, HW, L, r;              // r: radius of this lookup (the grid is laid out for the largest)
    int tap_stride, pix_stride;   // layout of out
    CellGrid g;
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
    int bin = -1;
    if (finite_ok) {
        const int u = ((int)floorf(cx) >> a.g.log_cx) - a.g.u_min;
        const int v = ((int)floorf(cy) >> a.g.log_cy) - a.g.v_min;
        if (u >= 0 && u < a.g.nbx && v >= 0 && v < a.g.nby) bin = corr_cell_id(a.g, b, u, v);
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
    if (!real) return;
    a.q_bin[q] = bin;
    a.q_rank[q] = rank;
    if (bin < 0) {   // out of range at every level: the whole output column of this query is zero
        float* o = a.out + (size_t)b * a.L * K * K * a.HW + (size_t)p * a.pix_stride;
        for (int t = 0; t < a.L * K * K; ++t) o[(size_t)t * a.tap_stride] = 0.0f;
    }
}

struct ScanArgs {
    int nbins, L, BN, r;
    CellGrid g;
    int Hl[CORR_MAX_L], Wl[CORR_MAX_L];
    int* bin_count;
    int* bin_off;
    int4* items;
    int* n_items;
    long long* stats;
};

// Single workgroup: exclusive scan of the counts (query offsets) and of the
// per-cell item counts, in tiles of 4096 cells (one int4 per thread, coalesced);
// writes the item list in cell order.
__global__ __launch_bounds__(1024) void bin_scan_kernel(ScanArgs a) {
    __shared__ int s_wc[16], s_wi[16];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    int carry_c = 0, carry_i = 0;
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
            a.bin_off[g] = coff;
            a.bin_count[g] = 0;                     // ready for the next lookup
            for (int s = 0; s < c[k]; s += CORR_GROUP)
                a.items[ioff++] = make_int4(g, coff + s, min(CORR_GROUP, c[k] - s), 0);
            coff += c[k];
        }
    }
    if (t == 0) { a.n_items[0] = carry_i; a.n_items[1] = carry_c; }   // items, binned queries
}

// On request only: work counters of the last binning, recomputed from the cell offsets.
__global__ __launch_bounds__(256) void bin_stats_kernel(ScanArgs a) {
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    const int lane = threadIdx.x & 63;
    const int K = 2 * a.r + 1;
    long long v[CORR_MAX_L][4] = {};
    if (g < a.nbins) {
        const int end = g + 1 < a.nbins ? a.bin_off[g + 1] : a.n_items[1];
        const int c = end - a.bin_off[g];
        if (c > 0) {
            int bb, u, w;
            corr_cell_coords(a.g, g, &bb, &u, &w);
            u += a.g.u_min; w += a.g.v_min;
            const int items_here = (c + CORR_GROUP - 1) / CORR_GROUP;
            const int pad_q = (c / CORR_GROUP) * CORR_GROUP + (((c % CORR_GROUP) + 15) & ~15);
#pragma unroll
            for (int l = 0; l < CORR_MAX_L; ++l) {
                if (l >= a.L) break;
                // window of this cell at level l and whether it touches the level at all
                const int wsx = max((1 << a.g.log_cx) >> l, 1) + K, wsy = max((1 << a.g.log_cy) >> l, 1) + K;
                const int xs = ((u << a.g.log_cx) >> l) - a.r, ys = ((w << a.g.log_cy) >> l) - a.r;
                if (xs + wsx - 1 >= 0 && xs <= a.Wl[l] - 1 && ys + wsy - 1 >= 0 && ys <= a.Hl[l] - 1) {
                    v[l][0] = items_here; v[l][1] = (long long)wsx * wsy * pad_q;
                    v[l][2] = (long long)wsx * wsy * c; v[l][3] = c;
                }
            }
        }
    }
#pragma unroll
    for (int l = 0; l < CORR_MAX_L; ++l)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            long long x = v[l][k];
#pragma unroll
            for (int d = 32; d > 0; d >>= 1) x += __shfl_xor(x, d, 64);
            if (lane == 0 && x) atomicAdd(reinterpret_cast<unsigned long long*>(&a.stats[8 + 4 * l + k]), (unsigned long long)x);
        }
}

__global__ __launch_bounds__(256) void bin_scatter_kernel(const int* __restrict__ q_bin,
                                                          const int* __restrict__ q_rank,
                                                          const int* __restrict__ bin_off,
                                                          int* __restrict__ perm, int BN) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= BN) return;
    const int bin = q_bin[i];
    if (bin >= 0) perm[bin_off[bin] + q_rank[i]] = i;
}

}  // namespace

static ScanArgs scan_args(corr_pyramid* p) {
    ScanArgs sc;
    sc.nbins = p->nbins; sc.L = p->L; sc.BN = p->B * p->H * p->W; sc.g = p->grid; sc.r = p->last_r;
    for (int l = 0; l < CORR_MAX_L; ++l) { sc.Hl[l] = p->Hl[l]; sc.Wl[l] = p->Wl[l]; }
    sc.bin_count = p->bin_count; sc.bin_off = p->bin_off; sc.items = p->items;
    sc.n_items = p->n_items; sc.stats = p->stats;
    return sc;
}

// stats[8 + 4*l + {0,1,2,3}] = items, issued and used point-queries, queries of level l
hipError_t launch_bin_stats(corr_pyramid* p, hipStream_t s) {
    hipError_t e = hipMemsetAsync(p->stats, 0, sizeof(long long) * CORR_NSTATS, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(bin_stats_kernel, dim3((p->nbins + 255) / 256), dim3(256), 0, s, scan_args(p));
    return hipGetLastError();
}

hipError_t launch_binning(corr_pyramid* p, const float* coords, int r, float* out, hipStream_t s) {
    const int HW = p->H * p->W, BN = p->B * HW;
    BinArgs a;
    a.coords = coords; a.out = out; a.B = p->B; a.HW = HW; a.L = p->L; a.r = r; a.g = p->grid;
    p->last_r = r;
    a.tap_stride = corr_tap_stride(p); a.pix_stride = corr_pix_stride(p, r);
    a.bin_count = p->bin_count; a.q_bin = p->q_bin; a.q_rank = p->q_rank;
    hipLaunchKernelGGL(bin_count_kernel, dim3((BN + 255) / 256), dim3(256), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    ScanArgs sc = scan_args(p);
    hipLaunchKernelGGL(bin_scan_kernel, dim3(1), dim3(1024), 0, s, sc);
    e = hipGetLastError();
    if (e != hipSuccess) return e;

    hipLaunchKernelGGL(bin_scatter_kernel, dim3((BN + 255) / 256), dim3(256), 0, s,
                       p->q_bin, p->q_rank, p->bin_off, p->perm, BN);
    return hipGetLastError();
}

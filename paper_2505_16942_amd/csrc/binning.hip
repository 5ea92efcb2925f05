// Per-lookup planning pass (paper: step a, "Setting Computation Mask" /
// "Implicit Computation Mask"): decide which blocks of the volume are computed.
//
// The paper groups source pixels by 8x8 source tile and lets each tile vote
// for the target blocks it needs.  Here the grouping is by *target*: a query
// belongs to the cell (floor(cx) >> 4, floor(cy) >> 3) of its level-0 target.
// Since floor(c / 2^l) == floor(c) >> l, the footprint origins of a cell's
// queries lie, at level l, in one aligned run of max(16 >> l, 1) x
// max(8 >> l, 1) pixels, so the cell owns one fixed window of
// (max(16 >> l, 1) + 2r + 1) x (max(8 >> l, 1) + 2r + 1) target pixels per
// level.  A work item is (cell, group of <= 128 of its queries); the blocks of
// the volume that get computed are exactly the items' window x group products,
// for every level.  Queries out of range at every level are written as zeros
// here and never reach the contraction.
//
// A counting sort over bins = (cell, source row mod 8), so that a cell's queries
// come out as runs of x-neighbouring source pixels, row after row: the lanes of
// one store of the block kernel's epilogue then hit few cache lines.
//   count   : bin id + slot per query (one atomic per run of equal bins among
//             consecutive lanes); the workgroup that finishes last also runs
//   scan    : cell and bin offsets, the item list
//   scatter : queries, and their coordinates, sorted by bin.
// Small inputs run all three steps in one workgroup.
#include "corr_internal.h"

namespace {

constexpr int SCAN_T = 1024;          // threads of a workgroup that scans
constexpr int SMALL_MAX_Q = 2;        // queries per thread of the one-workgroup path

struct BinArgs {
    const float* coords;   // [B][2][H*W]
    float* out;            // [B][L*K*K][H*W]
    int B, HW, W, L, r;           // r: radius of this lookup (the grid is laid out for the largest)
    int tap_stride, pix_stride;   // layout of out
    CellGrid g;
    BinWs ws;
};

// bin of query (b, p), or -1 when it is out of range at every level (then its output column is zeroed here)
__device__ __forceinline__ int query_bin(const BinArgs& a, int b, int p) {
    const float cx = a.coords[((size_t)b * 2 + 0) * a.HW + p];
    const float cy = a.coords[((size_t)b * 2 + 1) * a.HW + p];
    // comparisons are false for NaN, so non-finite coordinates are "not ok"
    const bool finite_ok = (fabsf(cx) <= CORR_COORD_LIMIT) && (fabsf(cy) <= CORR_COORD_LIMIT);
    int bin = -1;
    if (finite_ok) {
        const int u = ((int)floorf(cx) >> CORR_LOG_CX) - a.g.u_min;
        const int v = ((int)floorf(cy) >> CORR_LOG_CY) - a.g.v_min;
        if (u >= 0 && u < a.g.nbx && v >= 0 && v < a.g.nby)
            bin = corr_cell_id(a.g, b, u, v) * CORR_SUB + ((p / a.W) & (CORR_SUB - 1));
    }
    if (bin < 0) {
        const int K = 2 * a.r + 1;
        float* o = a.out + (size_t)b * a.L * K * K * a.HW + (size_t)p * a.pix_stride;
        for (int t = 0; t < a.L * K * K; ++t) o[(size_t)t * a.tap_stride] = 0.0f;
    }
    return bin;
}

// Neighbouring pixels mostly fall in the same bin: one atomic per run of equal bins among
// consecutive lanes, the rest of the run takes offsets.  Every lane of the wave must call this.
// In two halves, so that a caller with several queries per thread can have all its atomics in
// flight before it needs the first result.
struct RankTicket { int base, head_lane; };
__device__ __forceinline__ RankTicket take_rank_issue(int* bin_count, int bin) {
    const int lane = threadIdx.x & 63;
    const int prev = __shfl_up(bin, 1, 64);
    const bool head = (lane == 0) || (bin != prev);
    const unsigned long long heads = __ballot(head);
    const unsigned long long upto = (lane == 63) ? ~0ull : ((2ull << lane) - 1ull);
    RankTicket t;
    t.head_lane = 63 - __clzll((long long)(heads & upto));
    const unsigned long long above = heads & ~upto;
    const int next = above ? (__ffsll((long long)above) - 1) : 64;
    t.base = 0;
    if (head && bin >= 0) t.base = atomicAdd(&bin_count[bin], next - lane);
    return t;
}
__device__ __forceinline__ int take_rank_finish(const RankTicket& t) {
    const int lane = threadIdx.x & 63;
    return __shfl(t.base, t.head_lane, 64) + (lane - t.head_lane);
}
__device__ __forceinline__ int take_rank(int* bin_count, int bin) {
    return take_rank_finish(take_rank_issue(bin_count, bin));
}

// One workgroup of SCAN_T threads: exclusive scan of the bin counts (query offsets) and of the
// per-cell item counts, one cell per thread and tile; writes the item list in cell order and
// clears the counts for the next lookup.  Counts are read with device-scope atomic loads: they
// were produced by atomics of other workgroups, possibly on other XCDs.
__device__ void scan_cells(const BinWs& ws) {
    __shared__ int s_wc[SCAN_T / 64], s_wi[SCAN_T / 64];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    int carry_c = 0, carry_i = 0;
    const int ntiles = (ws.ncells + SCAN_T - 1) / SCAN_T;
    for (int tile = 0; tile < ntiles; ++tile) {
        const int cell = tile * SCAN_T + t;
        int c[CORR_SUB];
        int csum = 0;
#pragma unroll
        for (int k = 0; k < CORR_SUB; ++k) {
            c[k] = cell < ws.ncells ? __hip_atomic_load(&ws.bin_count[cell * CORR_SUB + k], __ATOMIC_RELAXED,
                                                        __HIP_MEMORY_SCOPE_AGENT) : 0;
            csum += c[k];
        }
        const int isum = (csum + CORR_GROUP - 1) / CORR_GROUP;
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
        for (int w = 0; w < SCAN_T / 64; ++w) {
            const int vc = s_wc[w], vi = s_wi[w];
            if (w < wave) { wc += vc; wi += vi; }
            tot_c += vc; tot_i += vi;
        }
        int coff = carry_c + wc + ci - csum, ioff = carry_i + wi + ii - isum;
        carry_c += tot_c; carry_i += tot_i;
        if (cell < ws.ncells) {
            for (int s = 0; s < csum; s += CORR_GROUP)
                ws.items[ioff++] = make_int4(cell, coff + s, min(CORR_GROUP, csum - s), 0);
#pragma unroll
            for (int k = 0; k < CORR_SUB; ++k) {
                ws.bin_off[cell * CORR_SUB + k] = coff;
                ws.bin_count[cell * CORR_SUB + k] = 0;          // ready for the next lookup
                coff += c[k];
            }
        }
    }
    if (t == 0) { ws.n_items[0] = carry_i; ws.n_items[1] = carry_c; ws.n_items[2] = 0; }
}

__global__ __launch_bounds__(SCAN_T) void bin_count_kernel(BinArgs a) {
    __shared__ int s_last;
    const int q = blockIdx.x * blockDim.x + threadIdx.x;   // b*HW + pixel
    const int BN = a.B * a.HW;
    const bool real = q < BN;                 // lanes past the end stay for the shuffles
    int bin = -1;
    if (real) { const int b = q / a.HW; bin = query_bin(a, b, q - b * a.HW); }
    const int rank = take_rank(a.ws.bin_count, bin);
    if (real) { a.ws.q_bin[q] = bin; a.ws.q_rank[q] = rank; }
    // The workgroup that arrives last scans.  Every thread has its atomic's result back before the
    // barrier, so the workgroup's additions are done when thread 0 takes the ticket; the scan reads
    // the counters with device-scope loads.
    __syncthreads();
    if (threadIdx.x == 0)
        s_last = __hip_atomic_fetch_add(&a.ws.n_items[2], 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT) == (int)gridDim.x - 1;
    __syncthreads();
    if (s_last) scan_cells(a.ws);
}

__global__ __launch_bounds__(256) void bin_scatter_kernel(BinArgs a) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= a.B * a.HW) return;
    const int bin = a.ws.q_bin[i];
    if (bin >= 0) {
        const int b = i / a.HW, p = i - b * a.HW;
        const int pos = a.ws.bin_off[bin] + a.ws.q_rank[i];
        a.ws.perm[pos] = i;
        a.ws.sorted_c[pos] = make_float2(a.coords[((size_t)b * 2 + 0) * a.HW + p], a.coords[((size_t)b * 2 + 1) * a.HW + p]);
    }
}

// Inputs of up to SCAN_T * SMALL_MAX_Q queries: count, scan and scatter in one workgroup, one launch.
__global__ __launch_bounds__(SCAN_T) void bin_small_kernel(BinArgs a) {
    const int BN = a.B * a.HW;
    int bin[SMALL_MAX_Q], rank[SMALL_MAX_Q];
    RankTicket ticket[SMALL_MAX_Q];
#pragma unroll
    for (int k = 0; k < SMALL_MAX_Q; ++k) {
        const int q = k * SCAN_T + threadIdx.x;
        bin[k] = -1;
        if (q < BN) { const int b = q / a.HW; bin[k] = query_bin(a, b, q - b * a.HW); }
    }
    // all of a thread's atomics are in flight before the first result is used
#pragma unroll
    for (int k = 0; k < SMALL_MAX_Q; ++k) {
        ticket[k].base = 0; ticket[k].head_lane = 0;
        if (k * SCAN_T < BN) ticket[k] = take_rank_issue(a.ws.bin_count, bin[k]);        // uniform condition
    }
#pragma unroll
    for (int k = 0; k < SMALL_MAX_Q; ++k) rank[k] = (k * SCAN_T < BN) ? take_rank_finish(ticket[k]) : 0;
    __syncthreads();                  // every atomic of this workgroup has returned
    scan_cells(a.ws);
    __syncthreads();                  // the offsets were written by threads of this workgroup
#pragma unroll
    for (int k = 0; k < SMALL_MAX_Q; ++k) {
        const int q = k * SCAN_T + threadIdx.x;
        if (q < BN && bin[k] >= 0) {
            const int b = q / a.HW, p = q - b * a.HW;
            const int pos = a.ws.bin_off[bin[k]] + rank[k];
            a.ws.perm[pos] = q;
            a.ws.sorted_c[pos] = make_float2(a.coords[((size_t)b * 2 + 0) * a.HW + p], a.coords[((size_t)b * 2 + 1) * a.HW + p]);
        }
    }
}

struct StatArgs {
    BinWs ws;
    CellGrid g;
    int L, r;
    int Hl[CORR_MAX_L], Wl[CORR_MAX_L];
};

// On request only: work counters of the last binning, recomputed from the cell offsets.
__global__ __launch_bounds__(256) void bin_stats_kernel(StatArgs a) {
    const int cell = blockIdx.x * blockDim.x + threadIdx.x;
    const int lane = threadIdx.x & 63;
    const int K = 2 * a.r + 1;
    long long v[CORR_MAX_L][4] = {};
    if (cell < a.ws.ncells) {
        const int end = cell + 1 < a.ws.ncells ? a.ws.bin_off[(cell + 1) * CORR_SUB] : a.ws.n_items[1];
        const int c = end - a.ws.bin_off[cell * CORR_SUB];
        if (c > 0) {
            int bb, u, w;
            corr_cell_coords(a.g, cell, &bb, &u, &w);
            u += a.g.u_min; w += a.g.v_min;
            const int items_here = (c + CORR_GROUP - 1) / CORR_GROUP;
            // columns the block kernel runs MFMAs for: a full group per item, half a group for an item of up to half
            const int rem = c % CORR_GROUP;
            const int pad_q = (c / CORR_GROUP) * CORR_GROUP + (rem == 0 ? 0 : rem > CORR_GROUP / 2 ? CORR_GROUP : CORR_GROUP / 2);
#pragma unroll
            for (int l = 0; l < CORR_MAX_L; ++l) {
                if (l >= a.L) break;
                // window of this cell at level l and whether it touches the level at all
                const int wsx = max((1 << CORR_LOG_CX) >> l, 1) + K, wsy = max((1 << CORR_LOG_CY) >> l, 1) + K;
                const int xs = ((u << CORR_LOG_CX) >> l) - a.r, ys = ((w << CORR_LOG_CY) >> l) - a.r;
                if (xs + wsx - 1 >= 0 && xs <= a.Wl[l] - 1 && ys + wsy - 1 >= 0 && ys <= a.Hl[l] - 1) {
                    v[l][0] = items_here; v[l][1] = (long long)((wsx * wsy + 15) & ~15) * pad_q;    // rows in blocks of 16
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
            if (lane == 0 && x) atomicAdd(reinterpret_cast<unsigned long long*>(&a.ws.stats[8 + 4 * l + k]), (unsigned long long)x);
        }
}

__global__ __launch_bounds__(256) void fill_i32_kernel(int* dst, int value, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = value;
}

}  // namespace

hipError_t launch_fill_i32(int* dst, int value, size_t n, hipStream_t s) {
    const int grid = (int)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
    hipLaunchKernelGGL(fill_i32_kernel, dim3(grid > 0 ? grid : 1), dim3(256), 0, s, dst, value, n);
    return hipGetLastError();
}

// stats[8 + 4*l + {0,1,2,3}] = items, issued and used point-queries, queries of level l
hipError_t launch_bin_stats(const corr_pyramid* p, const BinWs& ws, int r, hipStream_t s) {
    hipError_t e = launch_fill_i32(reinterpret_cast<int*>(ws.stats), 0, CORR_NSTATS * 2, s);
    if (e != hipSuccess) return e;
    StatArgs a;
    a.ws = ws; a.g = p->grid; a.L = p->L; a.r = r;
    for (int l = 0; l < CORR_MAX_L; ++l) { a.Hl[l] = p->Hl[l]; a.Wl[l] = p->Wl[l]; }
    hipLaunchKernelGGL(bin_stats_kernel, dim3((ws.ncells + 255) / 256), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_binning(const corr_pyramid* p, const BinWs& ws, const LookupArgs& q, hipStream_t s) {
    const int HW = p->H * p->W, BN = p->B * HW;
    BinArgs a;
    a.coords = q.coords; a.out = q.out; a.B = p->B; a.HW = HW; a.W = p->W; a.L = p->L; a.r = q.r; a.g = p->grid;
    a.tap_stride = corr_tap_stride(p, q); a.pix_stride = corr_pix_stride(p, q);
    a.ws = ws;
    if (BN <= SCAN_T * SMALL_MAX_Q) {
        hipLaunchKernelGGL(bin_small_kernel, dim3(1), dim3(SCAN_T), 0, s, a);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(bin_count_kernel, dim3((BN + SCAN_T - 1) / SCAN_T), dim3(SCAN_T), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(bin_scatter_kernel, dim3((BN + 255) / 256), dim3(256), 0, s, a);
    return hipGetLastError();
}

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


constexpr int SCAN_T = 1024;          // cells per tile of the scan; threads of the one-workgroup path
constexpr int COUNT_T = 1024;         // threads per workgroup of the count kernel
constexpr int SCAN_CPT = 1;           // cells per thread and tile when its last workgroup scans (2 was no faster, 4 costs
                                      // the kernel its two workgroups per CU)
constexpr int SMALL_MAX_Q = 2;        // queries per thread of the one-workgroup path

struct BinArgs {
    const float* coords;   // [B][2][H*W]
    int B, HW, W, L, r;           // r: radius of this lookup (the grid is laid out for the largest)
    CellGrid g;
    BinWs ws;
};

// bin of query (b, p), or -1 when it is out of range at every level (the block kernel's spare workgroups then write its zeros)
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

// One workgroup of T threads: exclusive scan of the bin counts (query offsets) and of the per-cell item
// counts, CPT consecutive cells per thread and tile of T * CPT cells; writes the item list in cell order and
// clears the counts for the next lookup.  The counts were produced by device-scope atomics of other
// workgroups, possibly on other XCDs: a caller that runs in the same kernel as those atomics puts an
// acquire fence in front (this XCD's L2 may hold stale copies of the lines).
template <int T, int CPT>
__device__ void scan_cells(const BinWs& ws) {
    static_assert(CORR_SUB == 8, "a cell's counters are two int4");
    __shared__ int s_wc[T / 64], s_wi[T / 64], s_tot[2];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    int carry_c = 0, carry_i = 0;
    const int ntiles = (ws.ncells + T * CPT - 1) / (T * CPT);
    for (int tile = 0; tile < ntiles; ++tile) {
        const int cell0 = (tile * T + t) * CPT;
        // a cell's counters are 32 contiguous bytes: two 16-byte loads per cell, all of a thread's in flight at once
        int4 lo[CPT], hi[CPT];
#pragma unroll
        for (int j = 0; j < CPT; ++j) {
            lo[j] = make_int4(0, 0, 0, 0); hi[j] = lo[j];
            if (cell0 + j < ws.ncells) {
                const int4* pc = reinterpret_cast<const int4*>(ws.bin_count + (size_t)(cell0 + j) * CORR_SUB);
                lo[j] = pc[0]; hi[j] = pc[1];
            }
        }
        int csum[CPT], isum[CPT], tc = 0, ti = 0;
#pragma unroll
        for (int j = 0; j < CPT; ++j) {
            csum[j] = lo[j].x + lo[j].y + lo[j].z + lo[j].w + hi[j].x + hi[j].y + hi[j].z + hi[j].w;
            isum[j] = (csum[j] + CORR_GROUP - 1) / CORR_GROUP;
            tc += csum[j]; ti += isum[j];
        }
        int ci = tc, ii = ti;                       // inclusive scan within the wave
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int vc = __shfl_up(ci, d, 64), vi = __shfl_up(ii, d, 64);
            if (lane >= d) { ci += vc; ii += vi; }
        }
        __syncthreads();                            // previous tile's shared values fully consumed
        if (lane == 63) { s_wc[wave] = ci; s_wi[wave] = ii; }
        __syncthreads();
        // the waves' totals are scanned by the first wave (a shuffle scan over T / 64 lanes): every thread
        // then needs two values only, which keeps this function's registers, and with them the registers of
        // the kernel that carries it, low
        if (wave == 0) {
            int vc = lane < T / 64 ? s_wc[lane] : 0, vi = lane < T / 64 ? s_wi[lane] : 0;
            const int oc = vc, oi = vi;
#pragma unroll
            for (int d = 1; d < T / 64; d <<= 1) {
                const int uc = __shfl_up(vc, d, 64), ui = __shfl_up(vi, d, 64);
                if (lane >= d) { vc += uc; vi += ui; }
            }
            if (lane < T / 64) { s_wc[lane] = vc - oc; s_wi[lane] = vi - oi; }       // exclusive prefix per wave
            if (lane == T / 64 - 1) { s_tot[0] = vc; s_tot[1] = vi; }
        }
        __syncthreads();
        const int wc = s_wc[wave], wi = s_wi[wave], tot_c = s_tot[0], tot_i = s_tot[1];
        int coff = carry_c + wc + ci - tc, ioff = carry_i + wi + ii - ti;
        carry_c += tot_c; carry_i += tot_i;
#pragma unroll
        for (int j = 0; j < CPT; ++j) {
            const int cell = cell0 + j;
            if (cell < ws.ncells) {
                for (int s = 0; s < csum[j]; s += CORR_GROUP)
                    ws.items[ioff++] = make_int4(cell, coff + s, min(CORR_GROUP, csum[j] - s), 0);
                // a cell's eight offsets and eight cleared counters: 16-byte stores (one store instruction per
                // 4-byte entry would be one memory request per lane and entry)
                const int o1 = coff + lo[j].x, o2 = o1 + lo[j].y, o3 = o2 + lo[j].z, o4 = o3 + lo[j].w;
                const int o5 = o4 + hi[j].x, o6 = o5 + hi[j].y, o7 = o6 + hi[j].z;
                int4* po = reinterpret_cast<int4*>(ws.bin_off + (size_t)cell * CORR_SUB);
                int4* pc = reinterpret_cast<int4*>(ws.bin_count + (size_t)cell * CORR_SUB);
                po[0] = make_int4(coff, o1, o2, o3);
                po[1] = make_int4(o4, o5, o6, o7);
                pc[0] = make_int4(0, 0, 0, 0);                   // ready for the next lookup
                pc[1] = make_int4(0, 0, 0, 0);
                coff += csum[j];
            }
        }
    }
    if (t == 0) { ws.n_items[0] = carry_i; ws.n_items[1] = carry_c; ws.n_items[2] = 0; }
    if (t < CORR_NTICKETS) ws.n_items[4 + t * CORR_TICKET_STRIDE] = 0;              // tickets ready for the next lookup
}

__global__ __launch_bounds__(COUNT_T) void bin_count_kernel(BinArgs a) {
    __shared__ int s_last;
    const int q = blockIdx.x * blockDim.x + threadIdx.x;   // b*HW + pixel
    const int BN = a.B * a.HW;
    const bool real = q < BN;                 // lanes past the end stay for the shuffles
    int bin = -1;
    const int b = real ? q / a.HW : 0, p = real ? q - b * a.HW : 0;
    if (real) bin = query_bin(a, b, p);
    const int rank = take_rank(a.ws.bin_count, bin);
    if (real) { a.ws.q_bin[q] = bin; a.ws.q_rank[q] = rank; }
    // The workgroup that arrives last scans.  Every thread has its atomic's result back before the
    // barrier: the workgroup's additions have been performed at the device's coherence point when thread 0
    // takes the ticket, and the scan reads the counters there too (device-scope atomic loads).  Counters and
    // ticket are only ever touched by device-scope atomics, so the ticket needs no fence of its own; a
    // release/acquire here would write back and invalidate the XCD's whole L2 once per workgroup, which is
    // what this kernel's time used to be (0.14 ms of it at 518 k queries).
    __syncthreads();
    if (threadIdx.x == 0) {
        // Two-stage sign-off: atomics on one address are served one after the other (50..80 ns each here), so
        // the workgroups spread over CORR_NTICKETS sub-tickets and only the last one on each takes the top one.
        const int sub = blockIdx.x % CORR_NTICKETS;
        const int on_sub = ((int)gridDim.x - sub + CORR_NTICKETS - 1) / CORR_NTICKETS;
        const int subs = min((int)gridDim.x, CORR_NTICKETS);
        bool last = __hip_atomic_fetch_add(&a.ws.n_items[4 + sub * CORR_TICKET_STRIDE], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == on_sub - 1;
        if (last) last = __hip_atomic_fetch_add(&a.ws.n_items[2], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == subs - 1;
        s_last = last;
    }
    __syncthreads();
    if (s_last) {
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");          // once, in one workgroup: drop stale lines, then read normally
        scan_cells<COUNT_T, SCAN_CPT>(a.ws);
        __syncthreads();
    }
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
        const int b = q < BN ? q / a.HW : 0, p = q < BN ? q - b * a.HW : 0;
        if (q < BN) { bin[k] = query_bin(a, b, p); a.ws.q_bin[q] = bin[k]; }     // the block kernel looks for the queries without a bin
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
    scan_cells<SCAN_T, 1>(a.ws);
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
    a.coords = q.coords; a.B = p->B; a.HW = HW; a.W = p->W; a.L = p->L; a.r = q.r; a.g = p->grid;
    a.ws = ws;
    if (BN <= SCAN_T * SMALL_MAX_Q) {
        hipLaunchKernelGGL(bin_small_kernel, dim3(1), dim3(SCAN_T), 0, s, a);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(bin_count_kernel, dim3((BN + COUNT_T - 1) / COUNT_T), dim3(COUNT_T), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(bin_scatter_kernel, dim3((BN + 255) / 256), dim3(256), 0, s, a);
    return hipGetLastError();
}

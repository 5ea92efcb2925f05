// Internal declarations shared by the library's translation units (host side of
// the C ABI and the kernel launchers).  Not part of the public boundary.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "corr.h"
#include "corr_bench.h"

#define CORR_MAX_L 4
#define CORR_CHUNK 32          // channels per chunk plane of the split representation
#define CORR_GROUP 128         // queries per work item (four waves of 32)
#define CORR_BLOCK_MAX_D 256   // channels of query fragments a wave of the block kernel holds in registers at a time
#define CORR_R 4               // largest lookup radius; the cell grid is laid out for it
#define CORR_LOG_CX 4          // target cell: 2^LOG_CX x 2^LOG_CY level-0 pixels
#define CORR_LOG_CY 3
#define CORR_SUB 8             // sub-bins per cell: source row mod 8, so a cell's queries come as runs of source pixels, row by row
#ifndef CORR_LOG_TX
#define CORR_LOG_TX 2          // super-tile: 2^LOG_TX x 2^LOG_TY cells whose ids are consecutive
#endif
#ifndef CORR_LOG_TY
#define CORR_LOG_TY 3
#endif
#define CORR_TILE_CELLS (1 << (CORR_LOG_TX + CORR_LOG_TY))
#ifndef CORR_SPLIT_LEVELS_MAX_QUERIES
#define CORR_SPLIT_LEVELS_MAX_QUERIES 32000   // inputs up to this many queries may run an item's levels in workgroups of their own
#endif
#ifndef CORR_NUM_CU
#define CORR_NUM_CU 256                       // compute units of the chip this is written for
#endif
#define CORR_COORD_LIMIT 1048576.0f
#define CORR_NSTATS 24
#define CORR_NTICKETS 16       // the count kernel's workgroups sign off on one of these, so that no counter sees them all
#define CORR_TICKET_STRIDE 32  // ints between sub-tickets: one cache line each
#define CORR_NCOUNTERS (4 + CORR_NTICKETS * CORR_TICKET_STRIDE)

// Target-cell grid.  A query belongs to the cell (floor(cx) >> LOG_CX,
// floor(cy) >> LOG_CY).  Because floor(c / 2^l) == floor(c) >> l, all queries of
// a cell have, at every level l, footprint origins inside one aligned run of
// max(CX >> l, 1) x max(CY >> l, 1) level-l pixels, so one fixed window per
// level serves the whole cell.
struct CellGrid {
    int u_min, v_min;      // cell coordinates of grid entry (0, 0); may be negative
    int nbx, nby;          // cells per axis (covers every query that is in range at some level)
    int tnx, tny;          // super-tiles per axis (grid padded up)
};

// Cell ids are super-tile major: the cells of a 4 x 8 super-tile (64 x 64 target pixels) are
// consecutive, so work items that run at the same time on one XCD cover a compact 2-D patch of
// the target image and find each other's window rows and columns in that XCD's L2.
__host__ __device__ static inline int corr_cell_id(const CellGrid& g, int b, int u, int v) {   // u, v grid-relative
    return (((b * g.tny + (v >> CORR_LOG_TY)) * g.tnx + (u >> CORR_LOG_TX)) << (CORR_LOG_TX + CORR_LOG_TY)) +
           ((v & ((1 << CORR_LOG_TY) - 1)) << CORR_LOG_TX) + (u & ((1 << CORR_LOG_TX) - 1));
}
__host__ __device__ static inline void corr_cell_coords(const CellGrid& g, int id, int* b, int* u, int* v) {
    const int tile = id >> (CORR_LOG_TX + CORR_LOG_TY), in = id & (CORR_TILE_CELLS - 1);
    *u = ((tile % g.tnx) << CORR_LOG_TX) + (in & ((1 << CORR_LOG_TX) - 1));
    *v = (((tile / g.tnx) % g.tny) << CORR_LOG_TY) + (in >> CORR_LOG_TX);
    *b = tile / (g.tnx * g.tny);
}

// Which work item workgroup w of the block kernel takes.  Workgroup w runs on XCD w % 8; items are dealt to
// the XCDs in runs of CORR_XCD_RUN consecutive items (neighbouring cells share window rows and columns, so
// they should share an L2), round robin, so that cheap border regions do not all land on one XCD.  On a grid
// that is a multiple of 8 * CORR_XCD_RUN workgroups (corr_block_grid) this is a permutation of the grid.
#ifndef CORR_XCD_RUN
#define CORR_XCD_RUN 32
#endif
__host__ __device__ static inline int corr_item_of_workgroup(int w) {
    const int j = w >> 3;
    return ((j / CORR_XCD_RUN) * 8 + (w & 7)) * CORR_XCD_RUN + j % CORR_XCD_RUN;
}
static inline int corr_block_grid(int max_items) {
    return (max_items + 8 * CORR_XCD_RUN - 1) / (8 * CORR_XCD_RUN) * (8 * CORR_XCD_RUN);
}

// Per-lookup planning workspace (device memory).  Sized by corr_ws_layout().
struct BinWs {
    int* bin_count;                // [nbins] zero between calls; bin = cell * CORR_SUB + (source row & (CORR_SUB - 1))
    int* bin_off;                  // [nbins] exclusive prefix of counts
    int* q_bin;                    // [B*H*W] bin id or -1
    int* q_rank;                   // [B*H*W] slot within the bin
    int* perm;                     // [B*H*W] queries sorted by bin
    float2* sorted_c;              // [B*H*W] their coordinates (x, y), in the same order
    int4* items;                   // [max_items] {cell id, first perm index, n queries, 0}
    int* n_items;                  // [CORR_NCOUNTERS]: items, binned queries, top ticket, 0, then CORR_NTICKETS sub-tickets CORR_TICKET_STRIDE ints apart
    long long* stats;              // [CORR_NSTATS]: 8+4*l+{0,1,2,3} per level
    int ncells, nbins, max_items;
};
// Byte offsets of the workspace arrays inside one allocation of `total` bytes.
struct WsLayout { size_t bin_count, bin_off, q_bin, q_rank, perm, sorted_c, items, n_items, stats, total; };

struct corr_pyramid {
    int B, H, W, D, L;
    unsigned reps;                 // representations allocated
    unsigned built;                // representations that hold the current pair (set by each build)
    int Hl[CORR_MAX_L], Wl[CORR_MAX_L];
    CellGrid grid;
    // CORR_REP_F32: channels-last fp32
    float* f1_nhwc;                // [B][H*W][D]
    float* f2_nhwc[CORR_MAX_L];    // [B][H_l*W_l][D]
    // CORR_REP_SPLIT: [D/32][P][64] bf16 (per 32-channel chunk 32 hi then 32 lo), P = all pixels
    // (f1: B*H*W; f2: every level, level-major then batch: pix_base[l] + b*H_l*W_l + y*W_l + x)
    uint16_t* f1_split;
    uint16_t* f2_split;
    // CORR_REP_BF16: [D/32][P][32] bf16 (the hi parts alone), same pixel order
    uint16_t* f1_hi;
    uint16_t* f2_hi;
    int f2_pix_base[CORR_MAX_L];   // first pixel of level l in a chunk plane
    int f2_pix_total;              // pixels per chunk plane
    // block-mode workspace (one allocation, carved by corr_ws_layout)
    void* ws_mem;
    BinWs ws;
    // CORR_MODE_FULLVOLUME cache (built lazily by the first full-volume lookup after a build)
    float* vol[CORR_MAX_L];        // [B][H*W][H_l*W_l]
    int vol_valid;
    size_t bytes;
};

// Fills `g` for level sizes (H >> l, W >> l), l < L, and the largest radius.
static inline void corr_fill_grid(CellGrid* g, int H, int W, int L) {
    const int r = CORR_R;
    const int m = L - 1;                       // the coarsest level reaches furthest outside
    // in range at level m  <=>  floor(c) >> m in [-r-1, W_m + r - 1]
    const int lo_x = (-r - 1) * (1 << m), hi_x = ((W >> m) + r) * (1 << m) - 1;
    const int lo_y = (-r - 1) * (1 << m), hi_y = ((H >> m) + r) * (1 << m) - 1;
    g->u_min = lo_x >> CORR_LOG_CX;            // arithmetic shift = floor
    g->v_min = lo_y >> CORR_LOG_CY;
    g->nbx = (hi_x >> CORR_LOG_CX) - g->u_min + 1;
    g->nby = (hi_y >> CORR_LOG_CY) - g->v_min + 1;
    g->tnx = (g->nbx + (1 << CORR_LOG_TX) - 1) >> CORR_LOG_TX;
    g->tny = (g->nby + (1 << CORR_LOG_TY) - 1) >> CORR_LOG_TY;
}
static inline int corr_ncells(const CellGrid& g, int B) { return B * CORR_TILE_CELLS * g.tnx * g.tny; }
static inline int corr_max_items(int BN, int ncells) { return BN / CORR_GROUP + (ncells < BN ? ncells : BN) + 1; }
static inline WsLayout corr_ws_layout(int BN, int ncells) {
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    WsLayout w;
    const size_t nbins = (size_t)ncells * CORR_SUB;
    size_t o = 0;
    w.bin_count = o; o = up(o + nbins * 4);
    w.bin_off = o; o = up(o + nbins * 4);
    w.q_bin = o; o = up(o + (size_t)BN * 4);
    w.q_rank = o; o = up(o + (size_t)BN * 4);
    w.perm = o; o = up(o + (size_t)BN * 4);
    w.sorted_c = o; o = up(o + (size_t)BN * 8);
    w.items = o; o = up(o + (size_t)corr_max_items(BN, ncells) * 16);
    w.n_items = o; o = up(o + CORR_NCOUNTERS * 4);
    w.stats = o; o = up(o + CORR_NSTATS * 8);
    w.total = o;
    return w;
}
static inline BinWs corr_ws_carve(void* mem, int BN, int ncells) {
    const WsLayout w = corr_ws_layout(BN, ncells);
    char* m = static_cast<char*>(mem);
    BinWs s;
    s.bin_count = reinterpret_cast<int*>(m + w.bin_count); s.bin_off = reinterpret_cast<int*>(m + w.bin_off);
    s.q_bin = reinterpret_cast<int*>(m + w.q_bin); s.q_rank = reinterpret_cast<int*>(m + w.q_rank);
    s.perm = reinterpret_cast<int*>(m + w.perm); s.sorted_c = reinterpret_cast<float2*>(m + w.sorted_c);
    s.items = reinterpret_cast<int4*>(m + w.items);
    s.n_items = reinterpret_cast<int*>(m + w.n_items); s.stats = reinterpret_cast<long long*>(m + w.stats);
    s.ncells = ncells; s.nbins = ncells * CORR_SUB; s.max_items = corr_max_items(BN, ncells);
    return s;
}

// What one lookup call asks for beyond the pyramid: passed down to the launchers, never stored.
struct LookupArgs {
    const float* coords;
    float* out;
    int r;          // radius of this lookup
    int nhwc;       // layout of out
    int prec;       // corr_precision
    int split_levels_max;   // block mode: inputs of up to this many queries run one workgroup per (item, level)
};
// Where tap t of pixel p of batch item b goes in `out`: b * taps * HW + t * tap_stride + p * pix_stride,
// with (tap_stride, pix_stride) = (HW, 1) for NCHW and (1, taps) for NHWC.
static inline int corr_tap_stride(const corr_pyramid* p, const LookupArgs& q) { return q.nhwc ? 1 : p->H * p->W; }
static inline int corr_pix_stride(const corr_pyramid* p, const LookupArgs& q) {
    return q.nhwc ? p->L * (2 * q.r + 1) * (2 * q.r + 1) : 1;
}

// launchers (each enqueues on `s` and returns hipGetLastError())
hipError_t launch_build_features(const float* nchw, int B, int D, int H, int W, int nlev,
                                 uint16_t* split, uint16_t* hi, float* const* nhwc, hipStream_t s);
hipError_t launch_copy_f32(float* dst, const float* src, size_t n, hipStream_t s);
hipError_t launch_fill_i32(int* dst, int value, size_t n, hipStream_t s);
hipError_t launch_binning(const corr_pyramid* p, const BinWs& ws, const LookupArgs& q, hipStream_t s);
hipError_t launch_bin_stats(const corr_pyramid* p, const BinWs& ws, int r, hipStream_t s);
// one instantiation of block.hip per lookup radius
hipError_t launch_block_r1(const corr_pyramid* p, const BinWs& ws, const LookupArgs& q, hipStream_t s);
hipError_t launch_block_r2(const corr_pyramid* p, const BinWs& ws, const LookupArgs& q, hipStream_t s);
hipError_t launch_block_r3(const corr_pyramid* p, const BinWs& ws, const LookupArgs& q, hipStream_t s);
hipError_t launch_block_r4(const corr_pyramid* p, const BinWs& ws, const LookupArgs& q, hipStream_t s);
hipError_t launch_ondemand(const corr_pyramid* p, const LookupArgs& q, hipStream_t s);
// gradient of the lookup (backward.hip): `ws` holds corr_backward_workspace_floats() floats
size_t corr_backward_workspace_floats(int B, int H, int W, int D, int L);      // the gradient arrays
size_t corr_backward_workspace_bytes_internal(int B, int H, int W, int D, int L);   // those and a planning workspace of its own
hipError_t launch_backward(const corr_pyramid* p, const float* coords, const float* d_out, int r,
                           float* d_fmap1, float* d_fmap2, float* ws, int form, int split_max, hipStream_t s);
hipError_t launch_fullvol_build(const corr_pyramid* p, hipStream_t s);
hipError_t launch_fullvol_sample(const corr_pyramid* p, const LookupArgs& q, hipStream_t s);

// Internal declarations shared by the library's translation units (host side of
// the C ABI and the kernel launchers).  Not part of the public boundary.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "corr.h"

#define CORR_MAX_L 4
#define CORR_CHUNK 32          // channels per chunk plane of the split representation
#define CORR_GROUP 64          // queries per work item
#define CORR_BLOCK_MAX_D 256   // channels of query fragments a wave of the block kernel holds in registers at a time
#define CORR_R 4               // largest lookup radius; the cell grid is laid out for it
#ifndef CORR_LOG_CX
#define CORR_LOG_CX 3          // target cell: 2^LOG_CX x 2^LOG_CY level-0 pixels
#endif
#define CORR_LOG_CY 3
#define CORR_COORD_LIMIT 1048576.0f
#define CORR_NSTATS 24
#define CORR_PROF_LOOKUPS 256

// Target-cell grid.  A query belongs to the cell (floor(cx) >> LOG_CX,
// floor(cy) >> LOG_CY).  Because floor(c / 2^l) == floor(c) >> l, all queries of
// a cell have, at every level l, footprint origins inside one aligned run of
// max(CX >> l, 1) x max(CY >> l, 1) level-l pixels, so one fixed window per
// level serves the whole cell.
struct CellGrid {
    int log_cx, log_cy;
    int u_min, v_min;      // cell coordinates of grid entry (0, 0); may be negative
    int nbx, nby;          // cells per axis (covers every query that is in range at some level)
    int tnx, tny;          // 8x8-cell super-tiles per axis (grid padded up)
    int r;
};

// Cell ids are super-tile major: the 64 cells of an 8x8 super-tile are consecutive, so work items
// that run at the same time on one XCD cover a compact 2-D patch of the target image and find
// each other's window rows and columns in that XCD's L2.
__host__ __device__ static inline int corr_cell_id(const CellGrid& g, int b, int u, int v) {   // u, v grid-relative
    return (((b * g.tny + (v >> 3)) * g.tnx + (u >> 3)) << 6) + ((v & 7) << 3) + (u & 7);
}
__host__ __device__ static inline void corr_cell_coords(const CellGrid& g, int id, int* b, int* u, int* v) {
    const int tile = id >> 6, in = id & 63;
    *u = (tile % g.tnx) * 8 + (in & 7);
    *v = ((tile / g.tnx) % g.tny) * 8 + (in >> 3);
    *b = tile / (g.tnx * g.tny);
}

struct corr_pyramid {
    int B, H, W, D, L;
    unsigned reps;                 // representations allocated
    unsigned built;                // representations that hold the current pair (set by each build)
    int Hl[CORR_MAX_L], Wl[CORR_MAX_L];
    CellGrid grid;
    int nbins;                     // B * 64 * tnx * tny
    int max_items;
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
    // block-mode workspace
    int* bin_count;                // [nbins] zero between calls
    int* bin_off;                  // [nbins] exclusive prefix of counts
    int* q_bin;                    // [B*H*W] cell id or -1
    int* q_rank;                   // [B*H*W] slot within the cell
    int* perm;                     // [B*H*W] queries sorted by cell
    int4* items;                   // [max_items] {cell id, first perm index, n queries, 0}
    int* n_items;                  // [4]: items, binned queries
    long long* stats;              // [CORR_NSTATS]: 0..4 totals, 8+4*l+{0,1,2,3} per level
    // CORR_MODE_FULLVOLUME cache
    float* vol[CORR_MAX_L];        // [B][H*W][H_l*W_l]
    int vol_valid;
    size_t bytes;
    int out_nhwc;                  // layout of `out` for the call being enqueued (set by corr_sample_layout)
    int last_r;                    // radius of the last block-mode lookup (for its work counters)
    // timing hook
    int prof_on, prof_n;
    hipEvent_t* prof_ev;           // [CORR_PROF_LOOKUPS][3]
};

// Fills `g` for level sizes (H >> l, W >> l), l < L, and radius r.
static inline void corr_fill_grid(CellGrid* g, int H, int W, int L, int r) {
    g->log_cx = CORR_LOG_CX; g->log_cy = CORR_LOG_CY; g->r = r;
    const int m = L - 1;                       // the coarsest level reaches furthest outside
    // in range at level m  <=>  floor(c) >> m in [-r-1, W_m + r - 1]
    const int lo_x = (-r - 1) * (1 << m), hi_x = ((W >> m) + r) * (1 << m) - 1;
    const int lo_y = (-r - 1) * (1 << m), hi_y = ((H >> m) + r) * (1 << m) - 1;
    g->u_min = lo_x >> g->log_cx;              // arithmetic shift = floor
    g->v_min = lo_y >> g->log_cy;
    g->nbx = (hi_x >> g->log_cx) - g->u_min + 1;
    g->nby = (hi_y >> g->log_cy) - g->v_min + 1;
    g->tnx = (g->nbx + 7) >> 3;
    g->tny = (g->nby + 7) >> 3;
}

// Where tap t of pixel p of batch item b goes in `out`: b * taps * HW + t * tap_stride + p * pix_stride,
// with (tap_stride, pix_stride) = (HW, 1) for NCHW and (1, taps) for NHWC.
static inline int corr_tap_stride(const corr_pyramid* p) { return p->out_nhwc ? 1 : p->H * p->W; }
static inline int corr_pix_stride(const corr_pyramid* p, int r) { return p->out_nhwc ? p->L * (2 * r + 1) * (2 * r + 1) : 1; }

// launchers (each enqueues on `s` and returns hipGetLastError())
hipError_t launch_build_features(const float* nchw, int B, int D, int H, int W, int nlev,
                                 uint16_t* split, uint16_t* hi, float* const* nhwc, hipStream_t s);
hipError_t launch_copy_f32(float* dst, const float* src, size_t n, hipStream_t s);
hipError_t launch_binning(corr_pyramid* p, const float* coords, int r, float* out, hipStream_t s);
hipError_t launch_bin_stats(corr_pyramid* p, hipStream_t s);
// one instantiation of block.hip per lookup radius
hipError_t launch_block_r1(corr_pyramid* p, const float* coords, int prec, float* out, hipStream_t s);
hipError_t launch_block_r2(corr_pyramid* p, const float* coords, int prec, float* out, hipStream_t s);
hipError_t launch_block_r3(corr_pyramid* p, const float* coords, int prec, float* out, hipStream_t s);
hipError_t launch_block_r4(corr_pyramid* p, const float* coords, int prec, float* out, hipStream_t s);
hipError_t launch_ondemand(corr_pyramid* p, const float* coords, int r, float* out, hipStream_t s);
hipError_t launch_fullvol_build(corr_pyramid* p, hipStream_t s);
hipError_t launch_fullvol_sample(corr_pyramid* p, const float* coords, int r, float* out, hipStream_t s);

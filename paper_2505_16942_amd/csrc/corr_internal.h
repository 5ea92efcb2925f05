// Internal declarations shared by the library's translation units (host side of
// the C ABI and the kernel launchers).  Not part of the public boundary.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "corr.h"

#define CORR_MAX_L 4
#define CORR_CHUNK 32          // channels per chunk plane of the split representation
#define CORR_PAD 16            // window origin of cell 0 along an axis is -CORR_PAD
#define CORR_GROUP 64          // queries per work item
#define CORR_COORD_LIMIT 1048576.0f
#define CORR_NSTATS 24
#define CORR_PROF_LOOKUPS 256

// Geometry of one level: size, target-cell side (1 << shift), cell grid.
struct LevelGeom {
    int H, W;          // level size
    int shift;         // cell side b = 1 << shift
    int nbx, nby;      // cells per axis
    int bin_base;      // first global cell id of this level
};

struct corr_pyramid {
    int B, H, W, D, L;
    unsigned reps;
    LevelGeom lv[CORR_MAX_L];
    int nbins;                     // all levels, all batch items
    int max_items;
    // CORR_REP_F32: channels-last fp32
    float* f1_nhwc;                // [B][H*W][D]
    float* f2_nhwc[CORR_MAX_L];    // [B][H_l*W_l][D]
    // CORR_REP_SPLIT: [B][D/32][pixels][64] bf16, 32 hi then 32 lo per pixel and chunk
    uint16_t* f1_split;
    uint16_t* f2_split[CORR_MAX_L];
    // block-mode workspace
    int* bin_count;                // [nbins] zero between calls
    int* bin_off;                  // [nbins] exclusive prefix of counts
    int* q_bin;                    // [L][B*H*W] cell id or -1
    int* q_rank;                   // [L][B*H*W] slot within the cell
    int* perm;                     // [L*B*H*W] queries sorted by cell
    int4* items;                   // [max_items] {cell id, first perm index, n queries, level}
    int* level_item_off;           // [L+1] first item of each level, last = total
    long long* stats;              // [CORR_NSTATS]: 0..4 totals, 8+4*l+{0,1,2,3} per level
    // CORR_MODE_FULLVOLUME cache
    float* vol[CORR_MAX_L];        // [B][H*W][H_l*W_l]
    int vol_valid;
    size_t bytes;
    // timing hook
    int prof_on, prof_n;
    hipEvent_t* prof_ev;           // [CORR_PROF_LOOKUPS][L + 2]
};

static inline int corr_level_dim(int v, int l) { return v >> l; }

// launchers (each enqueues on `s` and returns hipGetLastError())
hipError_t launch_build_features(const float* nchw, int B, int D, int H, int W, int nlev,
                                 uint16_t* const* split, float* const* nhwc, hipStream_t s);
hipError_t launch_binning(corr_pyramid* p, const float* coords, int r, float* out, hipStream_t s);
hipError_t launch_block(corr_pyramid* p, const float* coords, int r, int prec, float* out, hipStream_t s,
                        hipEvent_t* level_done);
hipError_t launch_ondemand(corr_pyramid* p, const float* coords, int r, float* out, hipStream_t s);
hipError_t launch_fullvol_build(corr_pyramid* p, hipStream_t s);
hipError_t launch_fullvol_sample(corr_pyramid* p, const float* coords, int r, float* out, hipStream_t s);

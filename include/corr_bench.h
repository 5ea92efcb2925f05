/*
 * corr_bench.h - measurement and test hooks of libcorr_mi355x.so.  None of these is part of the
 * method's boundary (that is corr.h); benchmarks and tests use them to count work, time kernels,
 * calibrate counters and read back internal state.
 */
#ifndef CORR_MI355X_BENCH_H
#define CORR_MI355X_BENCH_H

#include "corr.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Counters of the last CORR_MODE_BLOCK call on this pyramid, recomputed from the cell offsets its
 * planning pass left in the workspace, for a lookup of radius r.  Synchronises `stream` and copies
 * them to the host.
 *   items            work items = (target cell, group of <= 128 of its queries) pairs
 *   query_levels     B*H*W*L
 *   null_query_levels  query-levels whose cell window lies wholly outside the level (written as zeros,
 *                      no contraction)
 *   mma_point_queries  sum over items of window points (padded to 16-row blocks) x the query columns the
 *                      kernel runs (128 per item, 64 for an item of up to 64 queries): the contraction
 *                      work actually issued is 2*D*mma_point_queries flop per bf16 term
 *   used_point_queries sum over items of window points x real queries
 */
typedef struct {
    int64_t items;
    int64_t query_levels;
    int64_t null_query_levels;
    int64_t mma_point_queries;
    int64_t used_point_queries;
    /* the same, per level (entries >= L are zero); level_queries = query-levels that reached the contraction */
    int64_t level_items[4];
    int64_t level_mma_point_queries[4];
    int64_t level_used_point_queries[4];
    int64_t level_queries[4];
} corr_block_stats;
corr_status corr_last_block_stats(const corr_pyramid* pyr, int r, corr_block_stats* stats, void* stream);

/*
 * Timing hook for benchmarks (process-wide).  While enabled, every CORR_MODE_BLOCK call records HIP
 * events on its stream before the planning pass, after it, and after the block kernel (up to 256
 * lookups between two reads; `dropped` counts the calls beyond that).  corr_profile_read waits for
 * the recorded events, returns the sums of elapsed milliseconds and the number of lookups they
 * cover, and resets.  Not thread-safe; leave it off outside measurements.
 */
typedef struct {
    int64_t lookups;
    int64_t dropped;
    double binning_ms;
    double block_ms;         /* contraction + epilogue kernel (all levels) */
} corr_profile;
corr_status corr_profile_enable(int enable);
corr_status corr_profile_read(corr_profile* prof);

/* Host-side test hook of the binning rule (no device work).  Queries are grouped by the cell
 * (floor(x) >> 4, floor(y) >> 3) of their level-0 target; for level l < L this returns the sides of a
 * cell in level-l pixels (max(16 >> l, 1), max(8 >> l, 1)), the window of target pixels a cell owns
 * at that level (cell + 2*4 + 1 per axis) and the number of cells per axis of the grid (it extends
 * past the image as far as the coarsest level is in range). */
corr_status corr_bin_geometry(int H, int W, int L, int l, int* cell_x, int* cell_y,
                              int* window_x, int* window_y, int* cells_x, int* cells_y);

/* Measurement aid: a plain grid-stride copy of n floats (device to device) on `stream`.  Profiling
 * runs use it as the kernel of known size against which the HBM byte counters are scaled. */
corr_status corr_copy_f32(float* dst, const float* src, size_t n, void* stream);

/*
 * Test hook: the plan the last CORR_MODE_BLOCK call on this pyramid left in its workspace, copied
 * to host buffers (synchronises `stream`).
 *   counts[2] : number of items, number of binned queries
 *   items     : up to items_cap entries of 4 ints {cell id, first index into perm, queries, 0}
 *   perm      : up to perm_cap entries: query indices b*H*W + y*W + x sorted by (cell, source row mod 8)
 * Returns CORR_ERR_INVALID_ARG if a buffer is too small for what the plan holds.
 */
corr_status corr_debug_read_plan(const corr_pyramid* pyr, int32_t* counts, int32_t* items, size_t items_cap,
                                 int32_t* perm, size_t perm_cap, void* stream);
/*
 * Test hook (process-wide): block-mode lookups of up to `max_queries` queries (B*H*W) are launched with the
 * kernel that can run an item's levels in workgroups of their own (it does so while the item count is small
 * enough: four ways up to 64 items, two ways up to 384, else all levels in one workgroup).  0 = never (the
 * one-workgroup-per-item kernel that large inputs take), -1 restores the default (32000), -2 / -4 = always two / four ways, whatever the size.  All forms give the same bits.
 * Returns the previous setting.  Not synchronised with lookups in flight on other threads.
 * corr_sample_backward splits an item's levels over workgroups up to sizes of its own (all levels apart up to 32000 queries, level 0 apart up to 40000); a setting
 * of 0 switches that off, every other setting leaves the gradient at its default.
 */
int corr_debug_set_level_split(int max_queries);
/*
 * Test and measurement hook (process-wide): which kernel corr_sample_backward runs.  CORR_BACKWARD_ITEMS (the
 * default): the forward pass's work items, both gradients as fp32 matrix-core contractions over an item's
 * windows.  CORR_BACKWARD_QUERIES: one wave per query on the vector ALU with a float atomic per footprint
 * point and channel (the earlier form; kept as a cross-check and as the slower side of the comparison).
 * Both give the same gradients up to fp32 summation order.  Returns the previous setting.
 */
#define CORR_BACKWARD_ITEMS 0
#define CORR_BACKWARD_QUERIES 1
int corr_debug_set_backward_form(int form);
/*
 * Test hook (host only, no GPU work): the block kernel's launch grid for a workspace that can hold
 * `max_items` work items, and which item each workgroup takes: map[w] for w < *grid.  Pass map = NULL
 * to get the grid size alone; CORR_ERR_INVALID_ARG if map_cap < *grid.
 */
corr_status corr_debug_item_map(int max_items, int32_t* map, size_t map_cap, int* grid);
/* Test hook: absolute cell coordinates (floor(x) >> 4, floor(y) >> 3) and batch item of a cell id. */
corr_status corr_debug_cell_coords(const corr_pyramid* pyr, int cell_id, int* b, int* u, int* v);
/*
 * Test hook: level `level` of fmap2 as the pyramid holds it (level = -1: fmap1), converted to fp32
 * channels-last [B][H_l*W_l][D] in the host buffer `dst` (synchronises `stream`).
 *   rep = CORR_REP_F32 : the fp32 copy;  CORR_REP_SPLIT : hi + lo;  CORR_REP_BF16 : the hi parts.
 */
corr_status corr_debug_read_level(const corr_pyramid* pyr, unsigned rep, int level, float* dst, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CORR_MI355X_BENCH_H */

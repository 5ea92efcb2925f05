/*
 * corr.h - C ABI of the MI355X correlation-lookup library (libcorr_mi355x.so).
 *
 * The operation is the multi-level all-pairs correlation lookup of RAFT as the
 * paper states it (Eq. 1, Sec. "Problem and Baseline Implementation"; levels
 * use average-pooled target features, Sec. "Efficient Correlation Volume
 * Sampler"): for every source pixel p of fmap1, every level l < L and every
 * integer offset (i, j) in [0, 2r]^2,
 *
 *   out[b, l*K*K + i*K + j, y, x] = bilinear sample of
 *        C_l(p; v, u) = <fmap1[b,:,y,x], f2_l[b,:,v,u]> / sqrt(D)   (0 outside the level)
 *   at  u = coords[b,0,y,x] / 2^l + (i - r),   v = coords[b,1,y,x] / 2^l + (j - r),
 *
 * K = 2r+1, f2_0 = fmap2, f2_l = 2x2 mean of f2_{l-1} with floor sizes.
 * Sampling is in pixel coordinates (align_corners=True) with zero padding.
 * Non-finite or |c| > 2^20 coordinates give zeros for that query.
 *
 * All pointers named "device" are HIP device pointers on the current device;
 * `stream` is a hipStream_t passed as void* (NULL = the default stream).
 * Every call only enqueues work on `stream` unless stated otherwise and returns
 * a corr_status; nothing throws across this boundary.
 */
#ifndef CORR_MI355X_H
#define CORR_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct corr_pyramid corr_pyramid;   /* opaque, library-owned */

typedef enum {
    CORR_OK = 0,
    CORR_ERR_INVALID_ARG = -1,   /* null pointer, non-positive size, empty level, mismatch with the pyramid */
    CORR_ERR_UNSUPPORTED = -2,   /* D, L or r outside what the kernels are built for */
    CORR_ERR_OOM = -3,           /* a device allocation failed or would not fit (see corr_full_volume_bytes) */
    CORR_ERR_HIP = -4,           /* a HIP call or kernel launch failed */
    CORR_ERR_MISSING_REP = -5,   /* the pyramid was built without the representation this mode reads */
    CORR_ERR_TOO_LARGE = -6      /* corr_sample_static: the input needs more than CORR_STATIC_SCRATCH_BYTES */
} corr_status;

/* How corr_sample_mode computes the lookup.  All three give the same `out`. */
typedef enum {
    CORR_MODE_BLOCK = 0,       /* partial block-sparse volume: queries binned by target cell, one MFMA
                                  contraction per (cell window x query group), bilinear epilogue.
                                  The paper's method (Sec. "Efficient Correlation Volume Sampler"). */
    CORR_MODE_ONDEMAND = 1,    /* Eq. 1 evaluated per query, nothing stored (the paper's "on-demand"). */
    CORR_MODE_FULLVOLUME = 2   /* dense volume of Eq. 2 + pooled volume pyramid, then sampling
                                  (the paper's "default"); allocates corr_full_volume_bytes(). */
} corr_mode;

/* Arithmetic of the block contraction. */
typedef enum {
    CORR_PREC_BF16X3 = 0,   /* each fp32 feature split into bf16 hi + lo; hi*hi + hi*lo + lo*hi on bf16 MFMA,
                               fp32 accumulate: meets the fp32 bound 1e-4 * max|C| */
    CORR_PREC_BF16 = 1      /* hi*hi only: the paper's own precision (bf16 inputs, fp32 accumulate);
                               bound 2e-2 * max|C| */
} corr_precision;

/* Feature representations a pyramid can hold (bit mask). */
#define CORR_REP_SPLIT 1u   /* bf16 hi/lo, 32-channel chunk planes: read by CORR_MODE_BLOCK */
#define CORR_REP_F32   2u   /* fp32 channels-last: read by CORR_MODE_ONDEMAND and CORR_MODE_FULLVOLUME */
#define CORR_REP_BF16  4u   /* bf16 hi only, 32-channel chunk planes of 64-byte records: half the bytes of
                               CORR_REP_SPLIT; read by CORR_MODE_BLOCK with CORR_PREC_BF16, which prefers it
                               and otherwise reads the hi halves of CORR_REP_SPLIT */

/*
 * Per image pair (paper: "Input Preprocessing"): re-lays fmap1 and builds levels 0..L-1 of fmap2
 * (2x2 mean pooling, fp32) in the representations asked for.
 *   fmap1, fmap2 : device, dense fp32 [B, D, H, W] (NCHW); read only during the enqueued work.
 *   *pyr         : NULL -> a pyramid is allocated (hipMalloc; synchronous) and returned;
 *                  non-NULL -> must have been created with the same B,H,W,D,L and a superset of
 *                  `reps`; its buffers are reused and nothing is allocated.  Representations not
 *                  named in this call keep the previous pair and are not read by later lookups
 *                  (those return CORR_ERR_MISSING_REP).
 *   reps         : mask of CORR_REP_*; corr_pyramid_build uses CORR_REP_SPLIT.
 * Limits: 1 <= L <= 4 with H >> (L-1) >= 1 and W >> (L-1) >= 1; D a multiple of 32, D <= 1024;
 * B*H*W*81*L < 2^31; with P = B * (pixels of all L levels): P*D < 2^30, P < 2^24, and B*H*W*D < 2^30
 * (32-bit offsets inside the stored representations).  Anything beyond returns CORR_ERR_UNSUPPORTED.
 * The library owns the pyramid; free it with corr_pyramid_destroy.
 */
corr_status corr_pyramid_build(const float* fmap1, const float* fmap2,
                               int B, int H, int W, int D, int L,
                               corr_pyramid** pyr, void* stream);
corr_status corr_pyramid_build_reps(const float* fmap1, const float* fmap2,
                                    int B, int H, int W, int D, int L, unsigned reps,
                                    corr_pyramid** pyr, void* stream);
/* Waits for the work enqueued on `stream` (the stream the pyramid's builds and lookups were
 * ordered on), then frees everything the pyramid owns.  NULL is accepted. */
corr_status corr_pyramid_destroy(corr_pyramid* pyr, void* stream);
/* Device bytes currently owned by the pyramid (features, workspace, cached dense volume). */
size_t corr_pyramid_bytes(const corr_pyramid* pyr);

/*
 * Per lookup (paper: steps a-c of "Efficient Correlation Volume Sampler").
 *   fmap1   : device pointer given to corr_pyramid_build for this pyramid; kept for signature
 *             fidelity, the library reads its own re-laid copy (may be NULL).
 *   pyr     : pyramid built for the same B,H,W,D,L.
 *   coords  : device fp32 [B, 2, H, W]; channel 0 = x, 1 = y, absolute target position in
 *             level-0 pixels of fmap2.
 *   r       : lookup radius; 1 <= r <= 4 in every mode.
 *   out     : device fp32 [B, L*(2r+1)^2, H, W], fully overwritten (no need to zero it).
 * Nothing about a call is kept in the pyramid: radius, layout and precision travel with the
 * launch.  The pyramid is const here with one documented exception, a lazily built
 * representation: CORR_MODE_FULLVOLUME allocates and fills the dense volume on its first call
 * after a build and caches it in the pyramid until the next build or destroy.  Every other call
 * allocates nothing.  Work is enqueued on `stream`; calls that share a pyramid must be ordered
 * on one stream (they share its planning workspace).
 * corr_sample == corr_sample_mode(CORR_MODE_BLOCK, CORR_PREC_BF16X3, ...).
 */
corr_status corr_sample(const float* fmap1, const corr_pyramid* pyr, const float* coords,
                        int B, int H, int W, int D, int L, int r,
                        float* out, void* stream);
corr_status corr_sample_mode(corr_mode mode, corr_precision prec,
                             const float* fmap1, const corr_pyramid* pyr, const float* coords,
                             int B, int H, int W, int D, int L, int r,
                             float* out, void* stream);

/*
 * Gradient of the lookup with respect to the two feature maps (the paper names the backward pass as
 * future work, Sec. "Conclusion"; the operation is the derivative of Eq. 1 with the coordinates held
 * constant, as in RAFT, where they are detached):
 *     d_fmap1, d_fmap2 = d/d(fmap1, fmap2) of  sum(d_out * corr_sample(fmap1, pyr(fmap2), coords)).
 *   pyr       : built for the pair with CORR_REP_F32 (else CORR_ERR_MISSING_REP); its fmap1 copy and its
 *               fmap2 levels are what the gradient is taken at.
 *   coords    : device, fp32 [B, 2, H, W], as for corr_sample.
 *   d_out     : device, fp32 [B, L*(2r+1)^2, H, W] (NCHW), read only.
 *   d_fmap1, d_fmap2 : device, fp32 [B, D, H, W], fully overwritten.  The gradient of the pooled levels
 *               is folded into d_fmap2 (adjoint of the 2x2 mean; a trailing odd row or column that the
 *               pooling dropped receives level 0's share only).
 *   workspace : device, at least corr_backward_workspace_bytes(B, H, W, D, L) bytes, 16-byte aligned
 *               (else CORR_ERR_INVALID_ARG), caller-owned; contents on entry are ignored, contents on return
 *               are scratch.  It holds the channels-last gradients of fmap1 (one array per level for inputs of
 *               up to 32000 queries, two up to 40000) and of every level of fmap2, and a planning
 *               workspace of the call's own: the pyramid is only read, so the call may run beside lookups
 *               on the same pyramid.
 * Enqueues kernels on `stream` and returns; allocates nothing.  The queries are binned into the forward
 * pass's work items (a target cell and up to 128 of its queries); per item and level both gradients are
 * fp32 matrix-core contractions over the item's window (inputs of up to 40000 queries run an item's levels
 * in workgroups of their own and sum their shares of d_fmap1 in level order).  fp32 throughout.  d_fmap1 has the same bits on
 * every call; d_fmap2 is accumulated with floating-point atomics, so two calls agree to rounding, not bit
 * for bit.  Limits beyond corr_sample's: H*W*D*4 and H*W*(2r+1)^2*4 below 2^31 (one batch item's map and
 * one level's planes of d_out are addressed with 31-bit byte offsets), else CORR_ERR_UNSUPPORTED.
 */
size_t corr_backward_workspace_bytes(int B, int H, int W, int D, int L);
corr_status corr_sample_backward(const corr_pyramid* pyr, const float* coords, const float* d_out,
                                 int B, int H, int W, int D, int L, int r,
                                 float* d_fmap1, float* d_fmap2, void* workspace, size_t workspace_bytes,
                                 void* stream);

/*
 * corr_sample for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same result and same kernels as
 * corr_sample (block mode, bf16x3, NCHW out), but the planning workspace of the lookup (bin
 * counters and offsets, 20 bytes per query, the item list) is not the pyramid's: it is a fixed
 * array of CORR_STATIC_SCRATCH_BYTES that the library's code object holds on every GPU it is loaded
 * on, until the process ends.  The call allocates and frees nothing and only enqueues kernels on
 * `stream`.
 *   limit   : inputs whose workspace exceeds the array return CORR_ERR_TOO_LARGE (it holds
 *             B*H*W up to about 190,000 queries: a 270 x 480 map, the 4K-input configuration, needs
 *             2.7 MB and fits; a 540 x 960 map needs 10.9 MB and does not).
 *   sharing : all calls on one GPU use that GPU's one array, which keeps the previous call's
 *             contents; the call clears the counters it needs at zero itself.  Calls that overlap
 *             on one GPU (different streams, or a graph replay beside an eager call) race.
 */
#define CORR_STATIC_SCRATCH_BYTES (4u << 20)
corr_status corr_sample_static(const float* fmap1, const corr_pyramid* pyr, const float* coords,
                               int B, int H, int W, int D, int L, int r,
                               float* out, void* stream);

/*
 * Output layout option (not in the paper; its kernel writes the layout RAFT's next
 * convolution reads, which is CORR_OUT_NCHW).  CORR_OUT_NHWC writes the same values as
 * out[b, y, x, l*(2r+1)^2 + i*(2r+1) + j] (channels last: the L*(2r+1)^2 taps of a query are
 * contiguous), which is what a channels-last convolution reads and what the block kernel
 * can store in whole cache lines.  Everything else is as for corr_sample_mode, which is
 * corr_sample_layout(mode, prec, CORR_OUT_NCHW, ...).
 */
typedef enum { CORR_OUT_NCHW = 0, CORR_OUT_NHWC = 1 } corr_out_layout;
corr_status corr_sample_layout(corr_mode mode, corr_precision prec, corr_out_layout layout,
                               const float* fmap1, const corr_pyramid* pyr, const float* coords,
                               int B, int H, int W, int D, int L, int r, float* out, void* hip_stream);

/* Exact size of the dense volume pyramid of Eq. 2: 4 * B * (H*W) * sum_l(H_l*W_l) bytes
 * (0 if a level is empty or L is out of range).  Pure host arithmetic. */
size_t corr_full_volume_bytes(int B, int H, int W, int L);
/*
 * Device bytes the library holds for one image pair in `mode` with lookup radius r, beyond the
 * caller's inputs and outputs (paper Eq. 4, "Memory Complexity Analysis": the extra space of the
 * method is linear in the number of pixels P; the dense volume of Eq. 2 is quadratic):
 *   CORR_MODE_BLOCK      re-laid bf16 hi/lo features of fmap1 and of every level of fmap2
 *                        (4*D bytes per pixel) + the planning workspace (cell counters, three ints
 *                        per query, the item list): O(P * (D + 1)), independent of r
 *   CORR_MODE_ONDEMAND   channels-last fp32 features (4*D bytes per pixel): O(P * D)
 *   CORR_MODE_FULLVOLUME the same + corr_full_volume_bytes(): O(P^2)
 * 0 for unsupported sizes.  Pure host arithmetic; matches what corr_pyramid_bytes() reports after
 * a build with the representation that mode reads (and, for FULLVOLUME, one lookup).
 */
size_t corr_workspace_bytes(corr_mode mode, int B, int H, int W, int D, int L, int r);

const char* corr_status_string(corr_status s);

#ifdef __cplusplus
}
#endif
#endif /* CORR_MI355X_H */

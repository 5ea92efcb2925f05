/*
 * CPU oracle for the multi-level correlation lookup.  TEST INFRASTRUCTURE ONLY:
 * it is imported by tests, by the smoke check and by the benchmark's
 * cpu_baseline leg, never by the product path, and shares no code with the
 * HIP kernels.
 *
 * What it computes is the plain definition, written out tap by tap in fp64:
 *
 *   - the operator is the paper's Eq. 1 (Sec. "Problem and Baseline
 *     Implementation"): for source pixel y and target x the set of dot products
 *     <F1_y, F2_{x+dx}>, ||dx||_inf <= r, sampled bilinearly at non-integer x;
 *   - levels are independent and use the average-pooled target features
 *     (Sec. "Efficient Correlation Volume Sampler", single-level remark, and
 *     Sec. "Implementation Details");
 *   - RAFT conventions the paper inherits by claiming the exact RAFT operator:
 *     scale 1/sqrt(D), pixel-coordinate bilinear sampling (align_corners=True)
 *     with zero padding, level coordinate = c / 2^l, tap channel = i*K + j with
 *     i the x offset and j the y offset (the channel rule of the paper's helper
 *     listing, "ry + rx * K"), levels concatenated finest first.
 *
 * Every tap evaluates its four corner dot products independently (the
 * on-demand definition); nothing is shared between taps, nothing is tiled.
 * The only preprocessing is a change of memory layout to channels-last fp64
 * so that a dot product walks contiguous memory; summation order is d = 0..D-1.
 *
 * Pins (tests/test_oracle_pins.py): brute-force full 4-D volume with pooled
 * volume + explicit zero padding, pooling linearity, integer coordinates,
 * all-ones closed form, delta/hat functions, x/y transpose symmetry,
 * out-of-bounds zeros, integer-shift translation.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int L;
    int H[16], W[16];
    double *lev[16];   /* lev[l]: [B][H_l][W_l][D] channels-last fp64 */
} pyr64;

int corr_oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Level sizes: floor halving, a trailing odd row/column is dropped. */
int corr_oracle_level_size(int H, int W, int l, int *Hl, int *Wl) {
    for (int k = 0; k < l; ++k) { H /= 2; W /= 2; }
    *Hl = H; *Wl = W;
    return (H > 0 && W > 0) ? 0 : -1;
}

static void pyr_free(pyr64 *p) {
    for (int l = 0; l < p->L; ++l) free(p->lev[l]);
}

/* f2^0 = fmap2; f2^l[i][j] = 1/4 (f2^{l-1}[2i][2j] + [2i][2j+1] + [2i+1][2j] + [2i+1][2j+1]). */
static int pyr_build(pyr64 *p, const float *fmap2, int B, int D, int H, int W, int L) {
    memset(p, 0, sizeof(*p));
    p->L = L;
    for (int l = 0; l < L; ++l) {
        if (corr_oracle_level_size(H, W, l, &p->H[l], &p->W[l]) != 0) return -1;
        p->lev[l] = (double *)malloc(sizeof(double) * (size_t)B * p->H[l] * p->W[l] * D);
        if (!p->lev[l]) return -2;
    }
    /* level 0: NCHW fp32 -> NHWC fp64 */
    for (int b = 0; b < B; ++b)
        for (int d = 0; d < D; ++d)
            for (int y = 0; y < H; ++y)
                for (int x = 0; x < W; ++x)
                    p->lev[0][(((size_t)b * H + y) * W + x) * D + d] =
                        (double)fmap2[(((size_t)b * D + d) * H + y) * W + x];
    for (int l = 1; l < L; ++l) {
        const int Hp = p->H[l - 1], Wp = p->W[l - 1], Hl = p->H[l], Wl = p->W[l];
        const double *src = p->lev[l - 1];
        double *dst = p->lev[l];
        for (int b = 0; b < B; ++b)
            for (int y = 0; y < Hl; ++y)
                for (int x = 0; x < Wl; ++x)
                    for (int d = 0; d < D; ++d) {
                        const size_t r0 = (((size_t)b * Hp + 2 * y) * Wp + 2 * x) * D + d;
                        const size_t r1 = (((size_t)b * Hp + 2 * y + 1) * Wp + 2 * x) * D + d;
                        dst[(((size_t)b * Hl + y) * Wl + x) * D + d] =
                            0.25 * (src[r0] + src[r0 + D] + src[r1] + src[r1 + D]);
                    }
    }
    return 0;
}

/* Pooled target features, for tests: out_l is [B][D][H_l][W_l] fp64 (NCHW),
 * levels concatenated in `out`. */
int corr_oracle_pyramid(const float *fmap2, int B, int D, int H, int W, int L, double *out) {
    pyr64 p;
    int rc = pyr_build(&p, fmap2, B, D, H, W, L);
    if (rc) { pyr_free(&p); return rc; }
    size_t off = 0;
    for (int l = 0; l < L; ++l) {
        const int Hl = p.H[l], Wl = p.W[l];
        for (int b = 0; b < B; ++b)
            for (int d = 0; d < D; ++d)
                for (int y = 0; y < Hl; ++y)
                    for (int x = 0; x < Wl; ++x)
                        out[off + (((size_t)b * D + d) * Hl + y) * Wl + x] =
                            p.lev[l][(((size_t)b * Hl + y) * Wl + x) * D + d];
        off += (size_t)B * D * Hl * Wl;
    }
    pyr_free(&p);
    return 0;
}

/* C^l(b; p; v,u) = <f1(p), f2^l(v,u)> / sqrt(D) inside the level, 0 outside. */
static double corr_at(const double *f1p, const pyr64 *p, int b, int l, long v, long u, int D, double scale) {
    if (v < 0 || u < 0 || v >= p->H[l] || u >= p->W[l]) return 0.0;
    const double *f2 = p->lev[l] + (((size_t)b * p->H[l] + v) * p->W[l] + u) * D;
    double s = 0.0;
    for (int d = 0; d < D; ++d) s += f1p[d] * f2[d];
    return s * scale;
}

/* One output scalar: batch b, query (y,x), level l, tap (i,j); i <-> x offset. */
static double one_tap(const double *f1nhwc, const pyr64 *p, const float *coords,
                      int b, int y, int x, int l, int i, int j,
                      int H, int W, int D, int r, double scale) {
    const double cx = (double)coords[(((size_t)b * 2 + 0) * H + y) * W + x];
    const double cy = (double)coords[(((size_t)b * 2 + 1) * H + y) * W + x];
    if (!isfinite(cx) || !isfinite(cy)) return 0.0;          /* reading: non-finite -> 0 */
    const double inv = ldexp(1.0, -l);
    const double sx = cx * inv + (double)(i - r);
    const double sy = cy * inv + (double)(j - r);
    if (fabs(sx) > 1e12 || fabs(sy) > 1e12) return 0.0;      /* far outside any level */
    const double fx0 = floor(sx), fy0 = floor(sy);
    const double wx = sx - fx0, wy = sy - fy0;
    const long x0 = (long)fx0, y0 = (long)fy0;
    const double *f1p = f1nhwc + (((size_t)b * H + y) * W + x) * D;
    const double c00 = corr_at(f1p, p, b, l, y0, x0, D, scale);
    const double c01 = corr_at(f1p, p, b, l, y0, x0 + 1, D, scale);
    const double c10 = corr_at(f1p, p, b, l, y0 + 1, x0, D, scale);
    const double c11 = corr_at(f1p, p, b, l, y0 + 1, x0 + 1, D, scale);
    return (1.0 - wx) * (1.0 - wy) * c00 + wx * (1.0 - wy) * c01
         + (1.0 - wx) * wy * c10 + wx * wy * c11;
}

static double *f1_to_nhwc(const float *fmap1, int B, int D, int H, int W) {
    double *f = (double *)malloc(sizeof(double) * (size_t)B * H * W * D);
    if (!f) return NULL;
    for (int b = 0; b < B; ++b)
        for (int d = 0; d < D; ++d)
            for (int y = 0; y < H; ++y)
                for (int x = 0; x < W; ++x)
                    f[(((size_t)b * H + y) * W + x) * D + d] =
                        (double)fmap1[(((size_t)b * D + d) * H + y) * W + x];
    return f;
}

/* Whole lookup.  out: [B][L*K*K][H][W] fp64, fully written. */
int corr_oracle_lookup(const float *fmap1, const float *fmap2, const float *coords,
                       int B, int H, int W, int D, int L, int r, double *out) {
    if (B <= 0 || H <= 0 || W <= 0 || D <= 0 || L <= 0 || L > 16 || r < 0) return -1;
    pyr64 p;
    int rc = pyr_build(&p, fmap2, B, D, H, W, L);
    if (rc) { pyr_free(&p); return rc; }
    double *f1 = f1_to_nhwc(fmap1, B, D, H, W);
    if (!f1) { pyr_free(&p); return -2; }
    const int K = 2 * r + 1;
    const double scale = 1.0 / sqrt((double)D);
    const long NQ = (long)B * H * W;
#pragma omp parallel for schedule(dynamic, 16)
    for (long q = 0; q < NQ; ++q) {
        const int b = (int)(q / ((long)H * W));
        const int y = (int)((q / W) % H);
        const int x = (int)(q % W);
        for (int l = 0; l < L; ++l)
            for (int i = 0; i < K; ++i)
                for (int j = 0; j < K; ++j) {
                    const size_t ch = (size_t)l * K * K + (size_t)i * K + j;
                    out[(((size_t)b * L * K * K + ch) * H + y) * W + x] =
                        one_tap(f1, &p, coords, b, y, x, l, i, j, H, W, D, r, scale);
                }
    }
    free(f1);
    pyr_free(&p);
    return 0;
}

/* Selected outputs only: idx[n] are flat indices into the [B][L*K*K][H][W]
 * output; vals[n] receives each one, computed on its own. */
int corr_oracle_lookup_points(const float *fmap1, const float *fmap2, const float *coords,
                              int B, int H, int W, int D, int L, int r,
                              const int64_t *idx, long n, double *vals) {
    if (B <= 0 || H <= 0 || W <= 0 || D <= 0 || L <= 0 || L > 16 || r < 0) return -1;
    pyr64 p;
    int rc = pyr_build(&p, fmap2, B, D, H, W, L);
    if (rc) { pyr_free(&p); return rc; }
    double *f1 = f1_to_nhwc(fmap1, B, D, H, W);
    if (!f1) { pyr_free(&p); return -2; }
    const int K = 2 * r + 1;
    const double scale = 1.0 / sqrt((double)D);
    const int64_t total = (int64_t)B * L * K * K * H * W;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 64)
    for (long k = 0; k < n; ++k) {
        int64_t t = idx[k];
        if (t < 0 || t >= total) { bad = 1; vals[k] = NAN; continue; }
        const int x = (int)(t % W); t /= W;
        const int y = (int)(t % H); t /= H;
        const int ch = (int)(t % ((int64_t)L * K * K));
        const int b = (int)(t / ((int64_t)L * K * K));
        const int l = ch / (K * K), i = (ch % (K * K)) / K, j = ch % K;
        vals[k] = one_tap(f1, &p, coords, b, y, x, l, i, j, H, W, D, r, scale);
    }
    free(f1);
    pyr_free(&p);
    return bad ? -3 : 0;
}

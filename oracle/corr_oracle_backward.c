/*
 * CPU oracle for the gradient of the multi-level correlation lookup with respect to the two feature
 * maps.  TEST INFRASTRUCTURE ONLY (see corr_oracle.c); shares no code with the HIP kernels.
 *
 * The paper names the backward pass as future work (Sec. "Conclusion"); what it has to compute is
 * fixed by the forward definition (Eq. 1 with the conventions listed in corr_oracle.c).  Each output
 * is a sum over four corners c of w_c * <f1(p), f2_l(q_c)> / sqrt(D) with weights w_c that depend on
 * the coordinates only, and the coordinates are constants (RAFT detaches them).  So for an upstream
 * gradient g = d_out[b, l*K*K + i*K + j, p]:
 *
 *     d f1(p)      += g * w_c / sqrt(D) * f2_l(q_c)          for every corner inside level l
 *     d f2_l(q_c)  += g * w_c / sqrt(D) * f1(p)
 *
 * and the pooled levels pass their gradient down the pyramid by the adjoint of the 2x2 mean with
 * floor sizes: d f2_{l-1}[2v+a][2u+b] += 1/4 d f2_l[v][u], a, b in {0, 1}; a trailing odd row or
 * column of level l-1 was dropped by the pooling and receives nothing from level l.
 * Written out tap by tap and corner by corner in fp64, single pass, no tiling.
 *
 * Pins (tests/test_oracle_backward_pins.py): the lookup is linear in each feature map, so for any
 * direction a, <d_out, lookup(a, f2)> = <d f1, a> and <d_out, lookup(f1, a)> = <d f2, a> with the
 * forward oracle on the left (random and one-hot directions, odd sizes, windows partly outside);
 * the r = 0, L = 1, integer-coordinate case written out in numpy.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* d_out: [B][L*K*K][H][W]; d_f1, d_f2: [B][D][H][W], overwritten.  All fp64 except the inputs. */
int corr_oracle_backward(const float *fmap1, const float *fmap2, const float *coords, const double *d_out,
                         int B, int H, int W, int D, int L, int r, double *d_f1, double *d_f2) {
    if (B <= 0 || H <= 0 || W <= 0 || D <= 0 || L <= 0 || L > 16 || r < 0) return -1;
    const int K = 2 * r + 1;
    const double scale = 1.0 / sqrt((double)D);
    int Hl[16], Wl[16];
    double *lev[16], *dlev[16];
    memset(lev, 0, sizeof(lev)); memset(dlev, 0, sizeof(dlev));
    int rc = 0;
    for (int l = 0; l < L; ++l) {
        Hl[l] = l ? Hl[l - 1] / 2 : H;
        Wl[l] = l ? Wl[l - 1] / 2 : W;
        if (Hl[l] <= 0 || Wl[l] <= 0) { rc = -1; goto done; }
        const size_t n = (size_t)B * Hl[l] * Wl[l] * D;
        lev[l] = (double *)malloc(sizeof(double) * n);
        dlev[l] = (double *)calloc(n, sizeof(double));
        if (!lev[l] || !dlev[l]) { rc = -2; goto done; }
    }
    /* target features of every level, channels-last: level 0 = fmap2, level l = 2x2 mean of level l-1 */
    for (int b = 0; b < B; ++b)
        for (int d = 0; d < D; ++d)
            for (int y = 0; y < H; ++y)
                for (int x = 0; x < W; ++x)
                    lev[0][(((size_t)b * H + y) * W + x) * D + d] = (double)fmap2[(((size_t)b * D + d) * H + y) * W + x];
    for (int l = 1; l < L; ++l)
        for (int b = 0; b < B; ++b)
            for (int v = 0; v < Hl[l]; ++v)
                for (int u = 0; u < Wl[l]; ++u)
                    for (int d = 0; d < D; ++d) {
                        const double *s = lev[l - 1] + ((size_t)b * Hl[l - 1] * Wl[l - 1]) * D + d;
                        const size_t w = (size_t)Wl[l - 1];
                        lev[l][(((size_t)b * Hl[l] + v) * Wl[l] + u) * D + d] =
                            0.25 * (s[((2 * v) * w + 2 * u) * D] + s[((2 * v) * w + 2 * u + 1) * D] +
                                    s[((2 * v + 1) * w + 2 * u) * D] + s[((2 * v + 1) * w + 2 * u + 1) * D]);
                    }
    memset(d_f1, 0, sizeof(double) * (size_t)B * D * H * W);
    for (int b = 0; b < B; ++b)
        for (int y = 0; y < H; ++y)
            for (int x = 0; x < W; ++x) {
                const double cx = (double)coords[(((size_t)b * 2 + 0) * H + y) * W + x];
                const double cy = (double)coords[(((size_t)b * 2 + 1) * H + y) * W + x];
                if (!isfinite(cx) || !isfinite(cy)) continue;            /* the forward value is the constant 0 */
                for (int l = 0; l < L; ++l)
                    for (int i = 0; i < K; ++i)
                        for (int j = 0; j < K; ++j) {
                            const double g = d_out[(((size_t)b * L * K * K + (size_t)l * K * K + (size_t)i * K + j) * H + y) * W + x];
                            const double sx = cx * ldexp(1.0, -l) + (double)(i - r);
                            const double sy = cy * ldexp(1.0, -l) + (double)(j - r);
                            if (fabs(sx) > 1e12 || fabs(sy) > 1e12) continue;
                            const double fx0 = floor(sx), fy0 = floor(sy);
                            const double wx = sx - fx0, wy = sy - fy0;
                            for (int cyi = 0; cyi < 2; ++cyi)
                                for (int cxi = 0; cxi < 2; ++cxi) {
                                    const long u = (long)fx0 + cxi, v = (long)fy0 + cyi;
                                    if (u < 0 || v < 0 || u >= Wl[l] || v >= Hl[l]) continue;     /* zero padding: no dependence */
                                    const double w = (cxi ? wx : 1.0 - wx) * (cyi ? wy : 1.0 - wy);
                                    const double gw = g * w * scale;
                                    const size_t q = (((size_t)b * Hl[l] + v) * Wl[l] + u) * D;
                                    for (int d = 0; d < D; ++d) {
                                        d_f1[(((size_t)b * D + d) * H + y) * W + x] += gw * lev[l][q + d];
                                        dlev[l][q + d] += gw * (double)fmap1[(((size_t)b * D + d) * H + y) * W + x];
                                    }
                                }
                        }
            }
    /* down the pyramid: adjoint of the 2x2 mean */
    for (int l = L - 1; l >= 1; --l)
        for (int b = 0; b < B; ++b)
            for (int v = 0; v < Hl[l]; ++v)
                for (int u = 0; u < Wl[l]; ++u)
                    for (int d = 0; d < D; ++d) {
                        const double t = 0.25 * dlev[l][(((size_t)b * Hl[l] + v) * Wl[l] + u) * D + d];
                        for (int a2 = 0; a2 < 2; ++a2)
                            for (int b2 = 0; b2 < 2; ++b2)
                                dlev[l - 1][(((size_t)b * Hl[l - 1] + 2 * v + a2) * Wl[l - 1] + 2 * u + b2) * D + d] += t;
                    }
    for (int b = 0; b < B; ++b)
        for (int d = 0; d < D; ++d)
            for (int y = 0; y < H; ++y)
                for (int x = 0; x < W; ++x)
                    d_f2[(((size_t)b * D + d) * H + y) * W + x] = dlev[0][(((size_t)b * H + y) * W + x) * D + d];
done:
    for (int l = 0; l < L; ++l) { free(lev[l]); free(dlev[l]); }
    return rc;
}

"""Error bounds the GPU parity tests use, derived from the arithmetic of each precision mode.

fp32-accurate paths (on-demand, full volume, block mode with the bf16 hi+lo split):
    |err| <= 1e-4 * max|C|,  max|C| = the largest magnitude in the oracle's output.

bf16 mode (block mode on the hi parts alone).  Each factor of a product a_i * b_i is rounded to the
nearest bf16 (8 significant bits, unit roundoff u = 2^-8), so the product carries a relative error
d_i, |d_i| <= 2u + u^2, the sum of two independent rounding errors.  A rounding error is about uniform
within half a unit in the last place, which over a binade is 0.41 u relative (rms), so d_i has
standard deviation about 0.6 u (a simulation with normal features gives 0.60 u, for independent and
for strongly correlated pairs alike).  The error of one correlation value is sum_i a_i b_i d_i / sqrt(D):
zero mean, standard deviation 0.6 u * sqrt(sum_i (a_i b_i)^2 / D).  It does not grow with |C|; it grows
with the rms of the products, and sum_i (a_i b_i)^2 <= sqrt(sum a_i^4 * sum b_i^4) bounds that by the
features' fourth moments.  With m4(f) = max over pixels of mean_i f_i^4 the bound used here is

    |err| <= 8 * 0.6 * u * (m4(fmap1) * m4(fmap2))^(1/4)  +  1e-4 * max|C|

eight standard deviations (outputs number up to 1.7e8) plus the fp32 path's own allowance.  Pooled
levels and the bilinear mix are convex combinations, which only lower the fourth moment, so level 0's
moments cover every level.
"""
import numpy as np

FP32_TOL = 1e-4
BF16_U = 2.0 ** -8


def fp32_bound(ref) -> float:
    return FP32_TOL * float(np.abs(ref).max())


def _m4(f) -> float:
    f = np.asarray(f, dtype=np.float64)                  # [B, D, H, W]
    return float(np.mean(f ** 4, axis=1).max())


def bf16_bound(fmap1, fmap2, ref) -> float:
    return 8.0 * 0.6 * BF16_U * (_m4(fmap1) * _m4(fmap2)) ** 0.25 + fp32_bound(ref)

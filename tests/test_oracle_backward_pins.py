"""Pins of the gradient oracle (oracle/corr_oracle_backward.c) against things other than itself.

The lookup is linear in fmap1 for fixed fmap2 and coordinates, and linear in fmap2 likewise.  So for any
direction a: sum(d_out * lookup(a, fmap2)) = sum(d_fmap1 * a) and sum(d_out * lookup(fmap1, a)) =
sum(d_fmap2 * a), with the already pinned FORWARD oracle on the left.  Random directions check everything
at once; one-hot directions read out single gradient entries (a wrong index, a dropped corner, a pooling
adjoint that spreads to the wrong pixels or to a dropped trailing row fails these).  A closed form for
r = 0, L = 1 and integer coordinates is written out in numpy."""
import numpy as np
import pytest

from oracle import corr_oracle as oracle
from paper_2505_16942_amd import synth

CASES = [
    # B, H, W, D, L, r, flow range
    (1, 9, 11, 8, 3, 2, 3.0),       # odd sizes: levels 9x11, 4x5, 2x2; trailing rows and columns dropped
    (2, 8, 12, 4, 2, 1, 6.0),       # batch; windows partly outside
    (1, 6, 6, 16, 1, 4, 2.0),       # one level, full radius on a small map: most taps outside
    (1, 16, 20, 8, 4, 4, 5.0),      # four levels
]


def _case(case, seed):
    B, H, W, D, L, r, fr = case
    f1, f2, c = synth.small_case(seed, B, H, W, D, flow_range=fr)
    K = 2 * r + 1
    rng = np.random.default_rng(seed)
    d_out = rng.standard_normal((B, L * K * K, H, W))
    return f1, f2, c, d_out, L, r


@pytest.mark.parametrize("case", CASES)
def test_adjoint_identity_random_directions(case):
    f1, f2, c, d_out, L, r = _case(case, 11 + case[1])
    d1, d2 = oracle.backward(f1, f2, c, d_out, L=L, r=r)
    rng = np.random.default_rng(5)
    for _ in range(3):
        a = rng.standard_normal(f1.shape).astype(np.float32)
        lhs1 = float((d_out * oracle.lookup(a, f2, c, L=L, r=r)).sum())
        lhs2 = float((d_out * oracle.lookup(f1, a, c, L=L, r=r)).sum())
        rhs1 = float((d1 * a).sum())
        rhs2 = float((d2 * a).sum())
        scale = float(np.abs(d_out).sum())
        assert abs(lhs1 - rhs1) <= 1e-11 * scale, (lhs1, rhs1)
        assert abs(lhs2 - rhs2) <= 1e-11 * scale, (lhs2, rhs2)


@pytest.mark.parametrize("case", CASES[:2])
def test_single_entries_against_the_forward_oracle(case):
    f1, f2, c, d_out, L, r = _case(case, 23 + case[1])
    d1, d2 = oracle.backward(f1, f2, c, d_out, L=L, r=r)
    B, D, H, W = f1.shape
    rng = np.random.default_rng(9)
    picks = [(0, 0, 0, 0), (B - 1, D - 1, H - 1, W - 1), (0, 1, H - 1, 0), (0, 0, 0, W - 1)]
    picks += [tuple(int(rng.integers(n)) for n in (B, D, H, W)) for _ in range(8)]
    for idx in picks:
        e = np.zeros(f1.shape, np.float32)
        e[idx] = 1.0
        want1 = float((d_out * oracle.lookup(e, f2, c, L=L, r=r)).sum())
        want2 = float((d_out * oracle.lookup(f1, e, c, L=L, r=r)).sum())
        assert abs(d1[idx] - want1) <= 1e-11 * max(1.0, abs(want1)), ("d_fmap1", idx)
        assert abs(d2[idx] - want2) <= 1e-11 * max(1.0, abs(want2)), ("d_fmap2", idx)


def test_radius_zero_one_level_integer_coordinates_closed_form():
    """out[b, 0, p] = <f1(p), f2(c(p))> / sqrt(D) for integer c inside the map, 0 outside."""
    B, H, W, D = 2, 7, 9, 5
    f1, f2, c = synth.small_case(77, B, H, W, D, flow_range=4.0, integer_coords=True)
    rng = np.random.default_rng(1)
    d_out = rng.standard_normal((B, 1, H, W))
    d1, d2 = oracle.backward(f1, f2, c, d_out, L=1, r=0)
    want1 = np.zeros((B, D, H, W))
    want2 = np.zeros((B, D, H, W))
    s = 1.0 / np.sqrt(D)
    for b in range(B):
        for y in range(H):
            for x in range(W):
                u, v = int(c[b, 0, y, x]), int(c[b, 1, y, x])
                if 0 <= u < W and 0 <= v < H:
                    want1[b, :, y, x] += d_out[b, 0, y, x] * s * f2[b, :, v, u].astype(np.float64)
                    want2[b, :, v, u] += d_out[b, 0, y, x] * s * f1[b, :, y, x].astype(np.float64)
    assert np.abs(d1 - want1).max() <= 1e-13
    assert np.abs(d2 - want2).max() <= 1e-13


def test_non_finite_coordinates_give_no_gradient():
    f1, f2, c, d_out, L, r = _case(CASES[1], 3)
    c[0, 0, 2, 3] = np.float32("nan")
    c[1, 1, 4, 5] = np.float32("inf")
    d1, d2 = oracle.backward(f1, f2, c, d_out, L=L, r=r)
    assert np.all(d1[0, :, 2, 3] == 0.0) and np.all(d1[1, :, 4, 5] == 0.0)
    a = np.random.default_rng(2).standard_normal(f1.shape).astype(np.float32)
    assert abs(float((d_out * oracle.lookup(f1, a, c, L=L, r=r)).sum()) - float((d2 * a).sum())) <= 1e-10 * np.abs(d_out).sum()

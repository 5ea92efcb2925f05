"""Host property tests of the target-cell binning rule the planning pass uses.

The rule: a query belongs to the cell (floor(x) >> 4, floor(y) >> 3) of its level-0 target (16 x 8
pixels); at level l the cell owns the window of `window` pixels per axis that starts at
((cell << 4) >> l) - r in x and ((cell << 3) >> l) - r in y.  The properties checked here are what makes the block contraction exact:
every grid point a query's taps read, at every level, lies inside its cell's window, and the grid
covers every query that is in range at some level.  Also the paper's own bound on how many
aligned blocks one footprint can touch (supplementary, "Memory Complexity Analysis").
"""
import math
import os

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
R = 4
LCX, LCY = 4, 3      # log2 of the cell sides


def _geom(H, W, L, l):
    from paper_2505_16942_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        pytest.skip("library not built")
    return binding.corr_bin_geometry(H, W, L, l)


@pytest.mark.parametrize("shape", [(46, 62, 4), (135, 240, 4), (33, 17, 3), (8, 8, 4), (540, 960, 4)])
def test_footprints_lie_inside_the_cell_window(shape):
    H, W, L = shape
    rng = np.random.default_rng(H * 1000 + W)
    n = 20000
    cx = rng.uniform(-60, W + 60, n).astype(np.float32)
    cy = rng.uniform(-60, H + 60, n).astype(np.float32)
    # also exact integers and cell borders
    cx[:200] = np.round(cx[:200]); cy[:200] = np.round(cy[:200])
    cx[200:300] = (np.arange(100) * 8).astype(np.float32) - 8
    u = np.floor(cx).astype(np.int64) >> LCX
    v = np.floor(cy).astype(np.int64) >> LCY
    m = L - 1
    for l in range(L):
        cell_x, cell_y, win_x, win_y, nx, ny = _geom(H, W, L, l)
        # first grid point of the footprint at level l (oracle's definition, fp64 on fp32 coords)
        ox = np.floor(cx.astype(np.float64) / 2 ** l).astype(np.int64) - R
        oy = np.floor(cy.astype(np.float64) / 2 ** l).astype(np.int64) - R
        xs = ((u << LCX) >> l) - R
        ys = ((v << LCY) >> l) - R
        # footprint = ox .. ox + 2R + 1 ; window = xs .. xs + win - 1
        assert np.all(ox >= xs) and np.all(ox + 2 * R + 1 <= xs + win_x - 1)
        assert np.all(oy >= ys) and np.all(oy + 2 * R + 1 <= ys + win_y - 1)
        assert np.all(ox - xs < cell_x) and np.all(oy - ys < cell_y)
    # grid coverage: a query in range at ANY level has a cell inside the grid
    u_min = (-(R + 1) * (1 << m)) >> LCX
    v_min = (-(R + 1) * (1 << m)) >> LCY
    _, _, _, _, nx, ny = _geom(H, W, L, 0)
    in_grid = (u - u_min >= 0) & (u - u_min < nx) & (v - v_min >= 0) & (v - v_min < ny)
    in_range_any = np.zeros(n, bool)
    for l in range(L):
        Hl, Wl = H >> l, W >> l
        ox = np.floor(cx.astype(np.float64) / 2 ** l).astype(np.int64) - R
        oy = np.floor(cy.astype(np.float64) / 2 ** l).astype(np.int64) - R
        in_range_any |= (ox + 2 * R + 1 >= 0) & (ox <= Wl - 1) & (oy + 2 * R + 1 >= 0) & (oy <= Hl - 1)
    assert np.all(in_grid[in_range_any])


def test_paper_block_bound_holds_for_cells():
    # a (K+1)-wide footprint touches at most floor((K + 2B - 1)/B) aligned B-blocks per axis
    golden = os.path.join(ROOT, "tests", "golden", "paper_block_bound.txt")
    rows = [l.split() for l in open(golden) if l.strip() and not l.startswith("#")]
    r, B, want = (int(x) for x in rows[0])
    K = 2 * r + 1
    per_axis = (K + 2 * B - 1) // B
    assert per_axis ** 2 == want
    for o in range(-40, 40):
        touched = {(o + t) // B for t in range(K + 1)}
        assert len(touched) <= per_axis
    # our window of cell + K points per axis is what ONE cell needs instead of per_axis blocks of B
    assert B + K < per_axis * B


def test_window_work_per_query_is_bounded():
    # window points per query-level: the contraction does at most this many dot products per
    # query-level, against 100 for a lone query
    pts = [(max(16 >> l, 1) + 9) * (max(8 >> l, 1) + 9) for l in range(4)]
    assert pts == [425, 221, 143, 110]
    assert sum(pts) / 4 < 225

"""GPU checks of two intermediate results the end-to-end parity tests only see indirectly, read back
through the library's test hooks: the pooled pyramid levels in each stored representation, against
the oracle's pyramid, and the plan the binning pass leaves in its workspace (item list and sorted
query list), against the binning rule written out on the host."""
import numpy as np
import pytest

from oracle import corr_oracle as oracle
from paper_2505_16942_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

R = 4
LCX, LCY, SUB, GROUP = 4, 3, 8, 128
COORD_LIMIT = 1048576.0


def _binding():
    from paper_2505_16942_amd import binding
    binding.load_library()
    return binding


@pytest.mark.parametrize("shape", [(2, 37, 53, 96, 4), (1, 21, 35, 64, 3), (1, 8, 8, 32, 4)])
def test_pyramid_levels_match_the_oracle(shape):
    """Every level of fmap2 (and fmap1) as the library stores it, level by level against the oracle's
    2x2-mean pyramid with floor sizes (odd trailing rows and columns dropped).
    fp32 copy: pooling in fp32, at most 3 roundings per level -> 4e-7 * max|f| per level, absolute.
    split: hi + lo reproduces the fp32 value to 2^-16 relative (bf16 hi, bf16 lo of the remainder).
    hi only: round-to-nearest bf16 (8 significant bits), 2^-8 relative."""
    B, H, W, D, L = shape
    b = _binding()
    dev = torch.device("cuda:0")
    f1, f2, _ = synth.small_case(500 + H, B, H, W, D)
    t1, t2 = torch.from_numpy(f1).to(dev), torch.from_numpy(f2).to(dev)
    pyr = b.corr_pyramid_build(t1, t2, L=L, reps=b.CORR_REP_SPLIT | b.CORR_REP_F32 | b.CORR_REP_BF16)
    ref = oracle.pyramid(f2, L)                        # fp64 [B, D, H_l, W_l] per level
    levels = [(-1, f1.astype(np.float64))] + list(enumerate(ref))
    for l, want in levels:
        want = np.transpose(want, (0, 2, 3, 1))        # channels-last like the hook
        if l >= 0:
            assert want.shape[1:3] == (H >> l, W >> l)
        scale = float(np.abs(want).max())
        fp32_tol = 4e-7 * scale * (max(l, 0) + 1)
        got = b.corr_debug_read_level(pyr, b.CORR_REP_F32, l).astype(np.float64)
        e32 = float(np.abs(got - want).max())
        got = b.corr_debug_read_level(pyr, b.CORR_REP_SPLIT, l).astype(np.float64)
        esp = float(np.abs(got - want).max())
        got = b.corr_debug_read_level(pyr, b.CORR_REP_BF16, l).astype(np.float64)
        ehi = float((np.abs(got - want) - 2.0 ** -8 * np.abs(want)).max())
        print("level %d %s: fp32 err %.2e (tol %.2e), split err %.2e (tol %.2e), hi excess over 2^-8|v| %.2e"
              % (l, want.shape, e32, fp32_tol, esp, fp32_tol + 2.0 ** -16 * scale, ehi), flush=True)
        assert e32 <= fp32_tol
        assert esp <= fp32_tol + 2.0 ** -16 * scale
        assert ehi <= fp32_tol
    pyr.destroy()


def _host_rule(c, H, W, L, geom0):
    """Cell of every query under the rule, or -1: (b, u, v) absolute cell coordinates."""
    B = c.shape[0]
    cx, cy = c[:, 0].reshape(B, -1), c[:, 1].reshape(B, -1)
    m = L - 1
    u_min = (-(R + 1) * (1 << m)) >> LCX
    v_min = (-(R + 1) * (1 << m)) >> LCY
    nx, ny = geom0[4], geom0[5]
    with np.errstate(invalid="ignore"):
        ok = (np.abs(cx) <= COORD_LIMIT) & (np.abs(cy) <= COORD_LIMIT)
    fx = np.where(ok, np.floor(np.where(ok, cx, 0)), 0).astype(np.int64)
    fy = np.where(ok, np.floor(np.where(ok, cy, 0)), 0).astype(np.int64)
    u, v = fx >> LCX, fy >> LCY
    ok &= (u - u_min >= 0) & (u - u_min < nx) & (v - v_min >= 0) & (v - v_min < ny)
    return ok, u, v


@pytest.mark.parametrize("case", [(2, 24, 40, 4, 9.0), (2, 40, 60, 4, 9.0), (1, 100, 130, 4, 30.0), (3, 64, 48, 3, 3.0)])
def test_binning_workspace_against_the_rule(case):
    """What the count / scan / scatter kernels leave behind, read back and checked against the rule
    evaluated on the host: every binned query is listed exactly once, in an item of the cell the
    rule gives it; queries the rule leaves out are not listed; items partition the list, hold 1..128
    queries, a cell's items are full except its last; inside a cell queries come by source row mod 8.
    The first case takes the single-workgroup path (at most 2048 queries), the others the
    count + scatter path."""
    B, H, W, L, fr = case
    b = _binding()
    dev = torch.device("cuda:0")
    f1, f2, c = synth.small_case(700 + H, B, H, W, 32, flow_range=fr)
    rng = np.random.default_rng(H)
    out_idx = rng.choice(H * W, size=H * W // 20, replace=False)          # 5 % strays, some far outside the grid
    c.reshape(B, 2, -1)[0, :, out_idx] = rng.uniform(-400, 400, (out_idx.size, 2)).astype(np.float32)
    c[B - 1, 0, 1, 2] = np.float32("nan")
    c[B - 1, 1, 3, 4] = np.float32("inf")
    c[0, 0, 5, 6] = np.float32(-2e6)
    t1, t2, tc = (torch.from_numpy(a).to(dev) for a in (f1, f2, c))
    pyr = b.corr_pyramid_build(t1, t2, L=L)
    b.corr_sample(t1, pyr, tc)
    items, perm = b.corr_debug_read_plan(pyr)
    geom0 = b.corr_bin_geometry(H, W, L, 0)
    ok, u, v = _host_rule(c, H, W, L, geom0)
    HW = H * W
    want = np.flatnonzero(ok.reshape(-1))
    print("case", case, "queries", B * HW, "binned", want.size, "items", len(items), flush=True)
    assert 0 < want.size < B * HW                                          # both kinds are present
    assert np.array_equal(np.sort(perm), want)                             # exactly the rule's queries, once each
    first, n = items[:, 1], items[:, 2]
    assert np.all(n >= 1) and np.all(n <= GROUP) and int(n.sum()) == perm.size
    assert first[0] == 0 and np.array_equal(first[1:], np.cumsum(n)[:-1])  # items partition the list in order
    cells = items[:, 0]
    assert np.all(np.diff(cells) >= 0)                                     # cell order
    same = cells[1:] == cells[:-1]
    assert np.all(n[:-1][same] == GROUP)                                   # only a cell's last item is partial
    coords_of = {}
    for k, cell in enumerate(cells):
        if cell not in coords_of:
            coords_of[cell] = b.corr_debug_cell_coords(pyr, int(cell))
        cb_, cu, cv = coords_of[cell]
        q = perm[first[k]:first[k] + n[k]]
        qb, qp = q // HW, q % HW
        assert np.all(qb == cb_) and np.all(u[qb, qp] == cu) and np.all(v[qb, qp] == cv), "item %d" % k
    # inside a cell: by source row mod 8 (a cell's items are consecutive)
    start = 0
    for cell in np.unique(cells):
        cnt = int(n[cells == cell].sum())
        q = perm[start:start + cnt]
        sub = ((q % HW) // W) & (SUB - 1)
        assert np.all(np.diff(sub) >= 0), "cell %d" % cell
        start += cnt
    st = b.corr_last_block_stats(pyr, 4)
    assert st["items"] == len(items)
    pyr.destroy()

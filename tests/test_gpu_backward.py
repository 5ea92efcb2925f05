"""GPU parity of the lookup's gradient (corr_sample_backward, through the C ABI) against the fp64 gradient
oracle, element by element on the same seeded inputs.

Bar: max|err| <= 1e-4 * max|gradient| per output (d_fmap1, d_fmap2).  The kernel works in fp32: an element of
d_fmap1 is a sum of up to L * 100 terms, an element of d_fmap2 a sum over every query whose footprint
covers the pixel (accumulated with atomics in arbitrary order, then a quarter per pooled level); both are
relative errors of a few 1e-6 of the sum of magnitudes, inside the bound by an order of magnitude."""
import numpy as np
import pytest

from oracle import corr_oracle as oracle
from paper_2505_16942_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu
TOL = 1e-4

CASES = [
    # B, H, W, D, L, r, flow range
    (1, 21, 35, 64, 3, 4, 7.0),       # odd level sizes: trailing rows and columns dropped by the pooling
    (2, 16, 24, 32, 4, 4, 12.0),      # batch, D smaller than a wave
    (1, 8, 8, 96, 4, 4, 3.0),         # level 3 is a single pixel; D not a multiple of 64
    (1, 19, 27, 160, 2, 2, 30.0),     # r = 2, many windows outside
    (1, 13, 17, 320, 4, 1, 5.0),      # r = 1, five channel slots per lane; a second, partly filled channel group
    (2, 40, 60, 64, 4, 4, 9.0),       # 4800 queries: the count + scatter binning path, items of every fill
    (1, 12, 20, 512, 3, 3, 4.0),      # r = 3, two full channel groups
    (1, 10, 14, 32, 1, 4, 3.0),       # a single level
]
FORMS = ["items", "items, all levels in one workgroup", "queries"]


@pytest.fixture(params=FORMS)
def form(request):
    """Every oracle comparison runs for both kernels behind the entry point: the work-item form on the matrix
    cores (the default; with an item's levels split over workgroups, as small inputs run, and in one workgroup,
    as large ones do) and the one-wave-per-query form."""
    from paper_2505_16942_amd import binding
    binding.load_library()
    prev = binding.corr_debug_set_backward_form(
        binding.CORR_BACKWARD_QUERIES if request.param == "queries" else binding.CORR_BACKWARD_ITEMS)
    # small inputs run an item's levels in workgroups of their own; the second form switches that off
    prev_split = binding.corr_debug_set_level_split(0 if "one workgroup" in request.param else -1)
    yield request.param
    binding.corr_debug_set_backward_form(prev)
    binding.corr_debug_set_level_split(prev_split)


def _binding():
    from paper_2505_16942_amd import binding
    binding.load_library()
    return binding


def _check(got, want, what):
    got = got.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got)), what + ": non-finite gradient (an element was not written?)"
    m = float(np.abs(want).max())
    err = float(np.abs(got - want).max())
    print("%s: max|err| = %.3e, max|grad| = %.3f, bound = %.3e" % (what, err, m, TOL * m), flush=True)
    assert err <= TOL * max(m, 1e-30), what


@pytest.mark.parametrize("case", CASES)
def test_gradients_match_the_oracle(case, form):
    B, H, W, D, L, r, fr = case
    print("case", case, "form", form, flush=True)
    b = _binding()
    dev = torch.device("cuda:0")
    f1, f2, c = synth.small_case(300 + H, B, H, W, D, flow_range=fr)
    c[0, :, 1, 2] = np.float32(-1e6)                   # out of range at every level: no gradient from it
    c[B - 1, 0, 3, 1] = np.float32("nan")
    K = 2 * r + 1
    d_out = np.random.default_rng(H).standard_normal((B, L * K * K, H, W)).astype(np.float32)
    want1, want2 = oracle.backward(f1, f2, c, d_out, L=L, r=r)
    t1, t2, tc, tg = (torch.from_numpy(a).to(dev) for a in (f1, f2, c, d_out))
    pyr = b.corr_pyramid_build(t1, t2, L=L, reps=b.CORR_REP_F32)
    g1 = torch.full((B, D, H, W), float("nan"), device=dev)
    g2 = torch.full((B, D, H, W), float("nan"), device=dev)
    ws = torch.full((b.corr_backward_workspace_bytes(B, H, W, D, L) // 4,), float("nan"), device=dev)   # contents ignored
    b.corr_sample_backward(pyr, tc, tg, r=r, d_fmap1=g1, d_fmap2=g2, workspace=ws)
    torch.cuda.synchronize()
    _check(g1, want1, "d_fmap1 %s" % (case,))
    _check(g2, want2, "d_fmap2 %s" % (case,))
    assert float(g1[0, :, 1, 2].abs().max()) == 0.0 and float(g1[B - 1, :, 3, 1].abs().max()) == 0.0
    # a second call on the same workspace (now holding the first call's leftovers) gives the same result to rounding
    h1, h2 = b.corr_sample_backward(pyr, tc, tg, r=r, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(h1, g1)                          # no atomics on this output, one writer per partial sum: same bits
    _check(h2, want2, "d_fmap2, second call %s" % (case,))
    pyr.destroy()


def test_backward_agrees_with_the_forward_kernel_by_the_adjoint_identity():
    """<d_out, lookup(a, f2)> = <d_fmap1, a> with the library's own forward on the left: ties the two
    directions of the library together at a size beyond the oracle's reach in a test (135 x 240, D = 256)."""
    b = _binding()
    dev = torch.device("cuda:0")
    cfg = synth.config("1080p")
    f1, f2 = synth.features(cfg)
    c = synth.coords(cfg)
    t1, t2, tc = (torch.from_numpy(a).to(dev) for a in (f1, f2, c))
    gen = torch.Generator(device=dev); gen.manual_seed(5)
    d_out = torch.randn((1, 324, 135, 240), device=dev, generator=gen)
    a = torch.randn(t1.shape, device=dev, generator=gen)
    pyr = b.corr_pyramid_build(t1, t2, L=4, reps=b.CORR_REP_F32 | b.CORR_REP_SPLIT)
    g1, g2 = b.corr_sample_backward(pyr, tc, d_out)
    pa = b.corr_pyramid_build(a, t2, L=4)               # the lookup of direction a against the same targets
    lhs1 = float((d_out.double() * b.corr_sample(a, pa, tc).double()).sum())
    rhs1 = float((g1.double() * a.double()).sum())
    pb = b.corr_pyramid_build(t1, a, L=4)               # and of the pair (f1, a)
    lhs2 = float((d_out.double() * b.corr_sample(t1, pb, tc).double()).sum())
    rhs2 = float((g2.double() * a.double()).sum())
    scale = float(d_out.abs().sum()) * 1e-7          # ~1e7 terms of size ~1: rounding of the two sides is far below this
    print("adjoint identity: fmap1 %.6f vs %.6f, fmap2 %.6f vs %.6f (tolerance %.3f)" % (lhs1, rhs1, lhs2, rhs2, scale), flush=True)
    assert abs(lhs1 - rhs1) <= scale and abs(lhs2 - rhs2) <= scale
    for p in (pyr, pa, pb):
        p.destroy()


@pytest.mark.parametrize("cfg_name,r", [("1080p", 4), ("1080p", 2), ("voronoi", 4), ("voronoi", 3)])
def test_the_two_forms_agree_at_benchmark_sizes(cfg_name, r):
    """The work-item form against the one-wave-per-query form at sizes with hundreds of items of every fill
    (135 x 240 and the batched 2 x 104 x 208 configuration, D = 256), at the largest radius and a smaller one:
    both sum the same fp32 products in different orders, so they agree to a few 1e-6 of the largest gradient;
    and the work-item form's d_fmap1 is the same bits on a second call."""
    b = _binding()
    dev = torch.device("cuda:0")
    cfg = synth.config(cfg_name)
    B, H, W, L = cfg["B"], cfg["H"], cfg["W"], cfg["L"]
    K = 2 * r + 1
    f1, f2 = synth.features(cfg)
    t1, t2, tc = (torch.from_numpy(a).to(dev) for a in (f1, f2, synth.coords(cfg)))
    gen = torch.Generator(device=dev); gen.manual_seed(9)
    d_out = torch.randn((B, L * K * K, H, W), device=dev, generator=gen)
    pyr = b.corr_pyramid_build(t1, t2, L=L, reps=b.CORR_REP_F32)
    res = {}
    try:
        for name, form_id in (("items", b.CORR_BACKWARD_ITEMS), ("queries", b.CORR_BACKWARD_QUERIES)):
            b.corr_debug_set_backward_form(form_id)
            res[name] = b.corr_sample_backward(pyr, tc, d_out, r=r)
        b.corr_debug_set_backward_form(b.CORR_BACKWARD_ITEMS)
        again = b.corr_sample_backward(pyr, tc, d_out, r=r)
    finally:
        b.corr_debug_set_backward_form(b.CORR_BACKWARD_ITEMS)
    torch.cuda.synchronize()
    for i, what in enumerate(("d_fmap1", "d_fmap2")):
        m = float(res["queries"][i].abs().max())
        err = float((res["items"][i] - res["queries"][i]).abs().max())
        print("%s r=%d %s: max|items - queries| = %.3e, max|grad| = %.3f" % (cfg_name, r, what, err, m), flush=True)
        assert m > 0 and err <= 1e-5 * m
    assert torch.equal(again[0], res["items"][0])
    pyr.destroy()


def test_backward_replayed_from_a_hip_graph():
    """corr_sample_backward allocates nothing and clears what it accumulates into with kernels, so a caller may
    capture it (here two calls with different coordinates); every replay must give the eager d_fmap1 bit for bit and
    the eager d_fmap2 to rounding (its atomics are unordered), also with the program's own eager call in between."""
    b = _binding()
    dev = torch.device("cuda:0")
    B, H, W, D, L = 1, 30, 44, 64, 4
    f1, f2, c0 = synth.small_case(61, B, H, W, D, flow_range=9.0)
    _, _, c1 = synth.small_case(62, B, H, W, D, flow_range=9.0)
    t1, t2 = torch.from_numpy(f1).to(dev), torch.from_numpy(f2).to(dev)
    tcs = [torch.from_numpy(c0).to(dev), torch.from_numpy(c1).to(dev)]
    gen = torch.Generator(device=dev); gen.manual_seed(3)
    d_out = torch.randn((B, L * 81, H, W), device=dev, generator=gen)
    pyr = b.corr_pyramid_build(t1, t2, L=L, reps=b.CORR_REP_F32)
    ws = torch.empty(b.corr_backward_workspace_bytes(B, H, W, D, L) // 4, device=dev)
    g1 = [torch.empty_like(t1) for _ in range(2)]
    g2 = [torch.empty_like(t1) for _ in range(2)]

    def job():
        for t in range(2):
            b.corr_sample_backward(pyr, tcs[t], d_out, d_fmap1=g1[t], d_fmap2=g2[t], workspace=ws)

    job()
    torch.cuda.synchronize()
    e1, e2 = [x.clone() for x in g1], [x.clone() for x in g2]
    want = oracle.backward(f1, f2, c0, d_out.cpu().numpy(), L=L, r=4)
    _check(e1[0], want[0], "eager d_fmap1")
    _check(e2[0], want[1], "eager d_fmap2")
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            job()
    torch.cuda.synchronize()
    tol2 = 1e-5 * float(e2[0].abs().max())
    for rep in range(4):
        for x in g1 + g2:
            x.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for t in range(2):
            assert torch.equal(g1[t], e1[t]), "replay %d, d_fmap1 of call %d" % (rep, t)
            assert float((g2[t] - e2[t]).abs().max()) <= tol2, "replay %d, d_fmap2 of call %d" % (rep, t)
        b.corr_sample_backward(pyr, tcs[1], d_out, d_fmap1=g1[0], d_fmap2=g2[0], workspace=ws)   # eager work in between
        torch.cuda.synchronize()
        assert torch.equal(g1[0], e1[1])
    pyr.destroy()


@pytest.mark.parametrize("fill", ["nan", "far"])
def test_no_query_in_range_gives_zero_gradients(fill, form):
    """Coordinates that are all non-finite or far outside every level: the lookup is the constant 0, so both
    gradients are exactly 0 (no item exists; the outputs are still fully written)."""
    b = _binding()
    dev = torch.device("cuda:0")
    B, H, W, D, L = 2, 20, 28, 64, 4
    f1, f2, c = synth.small_case(81, B, H, W, D)
    t1, t2 = torch.from_numpy(f1).to(dev), torch.from_numpy(f2).to(dev)
    bad = torch.full((B, 2, H, W), float("nan") if fill == "nan" else 5000.0, device=dev)
    d_out = torch.ones((B, L * 81, H, W), device=dev)
    pyr = b.corr_pyramid_build(t1, t2, L=L, reps=b.CORR_REP_F32)
    g1 = torch.full((B, D, H, W), float("nan"), device=dev)
    g2 = torch.full((B, D, H, W), float("nan"), device=dev)
    b.corr_sample_backward(pyr, bad, d_out, d_fmap1=g1, d_fmap2=g2)
    torch.cuda.synchronize()
    assert torch.count_nonzero(g1).item() == 0 and torch.count_nonzero(g2).item() == 0
    assert not torch.isnan(g1).any() and not torch.isnan(g2).any()
    # and a normal call afterwards is unaffected
    tc = torch.from_numpy(c).to(dev)
    want = oracle.backward(f1, f2, c, d_out.cpu().numpy(), L=L, r=4)
    h1, h2 = b.corr_sample_backward(pyr, tc, d_out)
    torch.cuda.synchronize()
    _check(h1, want[0], "d_fmap1 after an empty call")
    _check(h2, want[1], "d_fmap2 after an empty call")
    pyr.destroy()


def test_backward_leaves_the_pyramids_plan_alone():
    """The gradient bins the queries in its own workspace: a lookup's plan in the pyramid (read back through the
    test hook) is the same before and after a backward call with other coordinates."""
    b = _binding()
    dev = torch.device("cuda:0")
    f1, f2, c = synth.small_case(77, 1, 40, 56, 64, flow_range=6.0)
    t1, t2, tc = (torch.from_numpy(a).to(dev) for a in (f1, f2, c))
    pyr = b.corr_pyramid_build(t1, t2, L=4, reps=b.CORR_REP_F32 | b.CORR_REP_SPLIT)
    b.corr_sample(t1, pyr, tc)
    items0, perm0 = b.corr_debug_read_plan(pyr)
    other = torch.from_numpy(synth.small_case(78, 1, 40, 56, 64, flow_range=15.0)[2]).to(dev)
    b.corr_sample_backward(pyr, other, torch.ones((1, 324, 40, 56), device=dev))
    torch.cuda.synchronize()
    items1, perm1 = b.corr_debug_read_plan(pyr)
    assert np.array_equal(items0, items1) and np.array_equal(perm0, perm1)
    pyr.destroy()


def test_backward_error_paths():
    b = _binding()
    dev = torch.device("cuda:0")
    f = torch.zeros((1, 32, 8, 8), device=dev)
    c = torch.zeros((1, 2, 8, 8), device=dev)
    g = torch.zeros((1, 324, 8, 8), device=dev)
    pyr = b.corr_pyramid_build(f, f, L=4)              # split representation only
    with pytest.raises(b.CorrError) as e:
        b.corr_sample_backward(pyr, c, g)
    assert e.value.status == b.CORR_ERR_MISSING_REP
    pyr.destroy()
    pyr = b.corr_pyramid_build(f, f, L=4, reps=b.CORR_REP_F32)
    small = torch.empty(16, device=dev)
    with pytest.raises(ValueError):
        b.corr_sample_backward(pyr, c, g, workspace=small)
    lib = b.load_library()
    st = lib.corr_sample_backward(pyr.handle, c.data_ptr(), g.data_ptr(), 1, 8, 8, 32, 4, 4, f.data_ptr(), f.data_ptr(),
                                  small.data_ptr(), 64, None)
    assert st == b.CORR_ERR_INVALID_ARG
    pyr.destroy()

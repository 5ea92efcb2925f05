"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (corr_pyramid_build with the split representation, then corr_sample in block
mode on the current stream).  The fp64 oracle is fast enough on the host to check EVERY output
of every configuration, so nothing here is sampled.

Bar: max|err| <= 1e-4 * max|C| (max|C| = largest magnitude of the oracle's output)."""
import time

import numpy as np
import pytest

from oracle import corr_oracle as oracle
from paper_2505_16942_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu
from tolerances import FP32_TOL, bf16_bound


def _cb():
    from paper_2505_16942_amd import binding
    binding.load_library()
    return binding


def _compare(out, ref, what, tol=FP32_TOL, bound=None):
    """bound: absolute; default tol * max|C|."""
    res = out.cpu().numpy()
    assert np.all(np.isfinite(res)), what + ": non-finite output"
    maxc = float(np.abs(ref).max())
    err = 0.0
    for ch0 in range(0, res.shape[1], 27):          # chunked to keep host memory flat
        d = np.abs(res[:, ch0:ch0 + 27].astype(np.float64) - ref[:, ch0:ch0 + 27]).max()
        err = max(err, float(d))
    if bound is None:
        bound = tol * maxc
    print("%s: max|err| = %.3e, max|C| = %.3f, bound = %.3e" % (what, err, maxc, bound), flush=True)
    assert err <= bound, what
    return err, maxc


def _setup(name):
    cb = _cb()
    cfg = synth.config(name)
    t0 = time.time()
    f1, f2 = synth.features(cfg)
    print("%s: inputs generated in %.1f s" % (name, time.time() - t0), flush=True)
    dev = torch.device("cuda:0")
    t1, t2 = torch.from_numpy(f1).to(dev), torch.from_numpy(f2).to(dev)
    return cb, cfg, f1, f2, t1, t2, dev


def test_1080p_all_modes_every_output():
    cb, cfg, f1, f2, t1, t2, dev = _setup("1080p")
    c = synth.coords(cfg)
    tc = torch.from_numpy(c).to(dev)
    ref = oracle.lookup(f1, f2, c, L=4, r=4)
    pyr = cb.corr_pyramid_build(t1, t2, L=4, reps=cb.CORR_REP_SPLIT | cb.CORR_REP_F32)
    out = torch.full((1, 324, 135, 240), float("nan"), device=dev)
    cb.corr_sample(t1, pyr, tc, out=out)
    _compare(out, ref, "1080p block bf16x3")
    st = cb.corr_last_block_stats(pyr)
    print("1080p stats", st, flush=True)
    assert st["query_levels"] == 135 * 240 * 4
    assert st["used_point_queries"] <= st["mma_point_queries"]
    # per query-level the contraction touches between 100 (a lone query's footprint) and 25 x 17 points
    live = st["query_levels"] - st["null_query_levels"]
    assert 100 * live <= st["used_point_queries"] <= 425 * live
    out.fill_(float("nan"))
    cb.corr_sample(t1, pyr, tc, out=out, prec=cb.CORR_PREC_BF16)
    # bf16 mode: absolute bound from the features' fourth moments; this input has max|C| ~ 17, where a bound
    # proportional to max|C| would be an order of magnitude looser than the error
    err16, maxc = _compare(out, ref, "1080p block bf16", bound=bf16_bound(f1, f2, ref))
    assert maxc > 10.0 and err16 > 1e-3        # the case is what it claims: large correlations, bf16-sized errors
    out.fill_(float("nan"))
    cb.corr_sample(t1, pyr, tc, out=out, mode=cb.CORR_MODE_ONDEMAND)
    _compare(out, ref, "1080p on-demand")
    out.fill_(float("nan"))
    before = pyr.bytes()
    cb.corr_sample(t1, pyr, tc, out=out, mode=cb.CORR_MODE_FULLVOLUME)
    _compare(out, ref, "1080p full volume")
    assert pyr.bytes() - before == cb.corr_full_volume_bytes(1, 135, 240, 4) == 5559840000
    pyr.destroy()


def test_4k_all_twelve_recurrent_lookups():
    """One pyramid build, then the twelve lookups of the recurrent pattern (the flow does a per-pixel random
    walk between them), each compared with the oracle on every output."""
    cb, cfg, f1, f2, t1, t2, dev = _setup("4k")
    pyr = cb.corr_pyramid_build(t1, t2, L=4)
    out = torch.empty((1, 324, 270, 480), device=dev)
    for t in range(12):
        c = synth.coords(cfg, t)
        ref = oracle.lookup(f1, f2, c, L=4, r=4)
        out.fill_(float("nan"))
        cb.corr_sample(t1, pyr, torch.from_numpy(c).to(dev), out=out)
        _compare(out, ref, "4k lookup %d" % t)
        del ref
    pyr.destroy()


def test_8k_every_output_and_full_volume_is_reported_not_run():
    cb, cfg, f1, f2, t1, t2, dev = _setup("8k")
    c = synth.coords(cfg)
    t0 = time.time()
    ref = oracle.lookup(f1, f2, c, L=4, r=4)
    print("8k oracle: %.1f s on %d threads" % (time.time() - t0, oracle.threads()), flush=True)
    pyr = cb.corr_pyramid_build(t1, t2, L=4, reps=cb.CORR_REP_SPLIT | cb.CORR_REP_F32)
    tc = torch.from_numpy(c).to(dev)
    out = torch.full((1, 324, 540, 960), float("nan"), device=dev)
    cb.corr_sample(t1, pyr, tc, out=out)
    _compare(out, ref, "8k block bf16x3")
    # twice on the same pyramid gives the same bits (no float atomics anywhere)
    out2 = torch.empty_like(out)
    cb.corr_sample(t1, pyr, tc, out=out2)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    del out2
    # the channels-last layout holds the same values (the launch configuration bench.py --out-layout nhwc times)
    out3 = torch.full((1, 540, 960, 324), float("nan"), dtype=torch.float32, device=out.device)
    cb.corr_sample(t1, pyr, tc, out=out3, layout=cb.CORR_OUT_NHWC)
    torch.cuda.synchronize()
    assert torch.equal(out, out3.permute(0, 3, 1, 2))
    del out3
    # the dense volume would need 1.43 TB: the library says so instead of trying
    with pytest.raises(cb.CorrError) as e:
        cb.corr_sample(t1, pyr, tc, out=out, mode=cb.CORR_MODE_FULLVOLUME)
    assert e.value.status == cb.CORR_ERR_OOM
    assert cb.corr_full_volume_bytes(1, 540, 960, 4) == 1427549184000
    pyr.destroy()


def test_voronoi_batched_block_and_ondemand():
    cb, cfg, f1, f2, t1, t2, dev = _setup("voronoi")
    c = synth.coords(cfg)
    ref = oracle.lookup(f1, f2, c, L=4, r=4)
    pyr = cb.corr_pyramid_build(t1, t2, L=4, reps=cb.CORR_REP_SPLIT | cb.CORR_REP_F32)
    tc = torch.from_numpy(c).to(dev)
    out = torch.full((2, 324, 270, 480), float("nan"), device=dev)
    cb.corr_sample(t1, pyr, tc, out=out)
    _compare(out, ref, "voronoi block bf16x3")
    out.fill_(float("nan"))
    cb.corr_sample(t1, pyr, tc, out=out, mode=cb.CORR_MODE_ONDEMAND)
    _compare(out, ref, "voronoi on-demand")
    # the dense volume of this configuration is 179 GB: it fits, so this mode runs here too
    need = cb.corr_full_volume_bytes(2, 270, 480, 4)
    print("voronoi full volume: %.1f GB" % (need / 1e9), flush=True)
    out.fill_(float("nan"))
    cb.corr_sample(t1, pyr, tc, out=out, mode=cb.CORR_MODE_FULLVOLUME)
    _compare(out, ref, "voronoi full volume")
    pyr.destroy()


@pytest.mark.parametrize("r", [1, 2, 3])
def test_1080p_smaller_radii(r):
    """Block mode (both precisions) and the on-demand mode at r < 4 on the full 1080p configuration."""
    cb, cfg, f1, f2, t1, t2, dev = _setup("1080p")
    c = synth.coords(cfg)
    # a few queries far outside and one without finite coordinates: null at this radius
    c[0, :, 7, 9] = np.float32(-300.0)
    c[0, 0, 100, 200] = np.float32("nan")
    tc = torch.from_numpy(c).to(dev)
    ref = oracle.lookup(f1, f2, c, L=4, r=r)
    K = 2 * r + 1
    pyr = cb.corr_pyramid_build(t1, t2, L=4, reps=cb.CORR_REP_SPLIT | cb.CORR_REP_F32)
    out = torch.full((1, 4 * K * K, 135, 240), float("nan"), device=dev)
    cb.corr_sample(t1, pyr, tc, r=r, out=out)
    _compare(out, ref, "1080p block bf16x3 r=%d" % r)
    out.fill_(float("nan"))
    cb.corr_sample(t1, pyr, tc, r=r, out=out, prec=cb.CORR_PREC_BF16)
    _compare(out, ref, "1080p block bf16 r=%d" % r, bound=bf16_bound(f1, f2, ref))
    out.fill_(float("nan"))
    cb.corr_sample(t1, pyr, tc, r=r, out=out, mode=cb.CORR_MODE_ONDEMAND)
    _compare(out, ref, "1080p on-demand r=%d" % r)
    pyr.destroy()


@pytest.mark.parametrize("D", [512, 320])
def test_more_channels_than_one_register_group(D):
    """D > 256 takes the block kernel's multi-pass path (query fragments of 256 channels at a time); checked
    here on a map of several hundred work items, 104 x 208, in both output layouts."""
    cb = _cb()
    dev = torch.device("cuda:0")
    B, H, W, L = 1, 104, 208, 4
    f1, f2, c = synth.small_case(900 + D, B, H, W, D, flow_range=20.0)
    ref = oracle.lookup(f1, f2, c, L=L, r=4)
    t1, t2, tc = (torch.from_numpy(a).to(dev) for a in (f1, f2, c))
    pyr = cb.corr_pyramid_build(t1, t2, L=L)
    out = torch.full((B, 324, H, W), float("nan"), device=dev)
    cb.corr_sample(t1, pyr, tc, out=out)
    _compare(out, ref, "D=%d block bf16x3" % D)
    st = cb.corr_last_block_stats(pyr)
    assert st["items"] > 150
    ocl = torch.full((B, H, W, 324), float("nan"), device=dev)
    cb.corr_sample(t1, pyr, tc, out=ocl, layout=cb.CORR_OUT_NHWC)
    assert torch.equal(ocl.permute(0, 3, 1, 2), out)
    out.fill_(float("nan"))
    cb.corr_sample(t1, pyr, tc, out=out, prec=cb.CORR_PREC_BF16)
    _compare(out, ref, "D=%d block bf16" % D, bound=bf16_bound(f1, f2, ref))
    pyr.destroy()

"""corr_sample_static (the entry point for callers that cannot allocate) against corr_sample:
same kernels on the library's fixed scratch array instead of the pyramid's workspace, so the
outputs must be identical; and against the oracle to the fp32 bar.  Two calls in a row, the
second with a smaller input (the array keeps the first call's contents)."""
import gc

import numpy as np
import pytest

from oracle import corr_oracle as oracle
from paper_2505_16942_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu
FP32_TOL = 1e-4


def _case(b, seed, B, H, W, D, L, fr):
    dev = torch.device("cuda:0")
    f1, f2, c = synth.small_case(seed, B, H, W, D, flow_range=fr)
    t1, t2, tc = (torch.from_numpy(a).to(dev) for a in (f1, f2, c))
    pyr = b.corr_pyramid_build(t1, t2, L=L)
    want = b.corr_sample(t1, pyr, tc)
    torch.cuda.synchronize()
    out = torch.full_like(want, float("nan"))
    gc.collect()                                   # leftovers of earlier tests must not be freed in between
    held, before = pyr.bytes(), torch.cuda.memory_allocated()
    b.corr_sample_static(t1, pyr, tc, out=out)
    torch.cuda.synchronize()
    assert pyr.bytes() == held and torch.cuda.memory_allocated() <= before
    assert torch.equal(out, want), "static-scratch lookup differs from corr_sample"
    ref = oracle.lookup(f1, f2, c, L=L, r=4)
    err = float(np.abs(out.cpu().numpy().astype(np.float64) - ref).max())
    maxc = float(np.abs(ref).max())
    print("static %dx%d: max|err| = %.3e, bound %.3e" % (H, W, err, FP32_TOL * maxc), flush=True)
    assert err <= FP32_TOL * maxc
    # once more on the same pyramid: the array now holds this call's own leftovers
    out.fill_(float("nan"))
    b.corr_sample_static(t1, pyr, tc, out=out)
    torch.cuda.synchronize()
    assert torch.equal(out, want)
    pyr.destroy()


def test_two_calls_in_a_row_second_smaller_and_the_size_limit():
    from paper_2505_16942_amd import binding as b
    b.load_library()
    _case(b, 301, 2, 96, 128, 64, 4, 20.0)      # 24,576 queries: the multi-workgroup planning path
    _case(b, 302, 1, 30, 44, 96, 3, 9.0)        # smaller: one-workgroup planning, other bin layout
    dev = torch.device("cuda:0")
    # the largest benchmark configuration that fits the array (270 x 480: 2.7 MB of workspace)
    g = torch.randn((1, 32, 270, 480), device=dev)
    cc = torch.rand((1, 2, 270, 480), device=dev) * 300.0
    pyr = b.corr_pyramid_build(g, g, L=4)
    assert torch.equal(b.corr_sample_static(g, pyr, cc), b.corr_sample(g, pyr, cc))
    pyr.destroy()
    # beyond the array: refused with its own status, nothing enqueued
    f = torch.zeros((1, 32, 540, 960), device=dev)
    pyr = b.corr_pyramid_build(f, f, L=4)
    c = torch.zeros((1, 2, 540, 960), device=dev)
    out = torch.empty((1, 324, 540, 960), device=dev)
    with pytest.raises(b.CorrError) as e:
        b.corr_sample_static(f, pyr, c, out=out)
    assert e.value.status == b.CORR_ERR_TOO_LARGE
    pyr.destroy()

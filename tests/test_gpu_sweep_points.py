"""Oracle parity at the shapes the sweep script times (paper: appendix table of the isolated sampling
benchmark, one variable at a time): widths 32..512 at 7W/16 rows and D = 256, and D = 64..1024 at width
256, on the inputs the sweep itself draws.  Block mode, both precisions."""
import numpy as np
import pytest

from oracle import corr_oracle as oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu
from tolerances import FP32_TOL, bf16_bound

POINTS = [(32, 256), (64, 256), (128, 256), (256, 256), (512, 256), (256, 64), (256, 128), (256, 512), (256, 1024)]


@pytest.mark.parametrize("point", POINTS)
def test_sweep_point_matches_the_oracle(point):
    from paper_2505_16942_amd import binding as cb
    from paper_2505_16942_amd import sweep
    cb.load_library()
    width, D = point
    H, W, f1, f2, cs = sweep._case(width, D, 7000 + width + D)
    assert (H, W) == (max(width * 7 // 16, 8), width)
    h1, h2, hc = f1.cpu().numpy(), f2.cpu().numpy(), cs[1].cpu().numpy()
    ref = oracle.lookup(h1, h2, hc, L=4, r=4)
    maxc = float(np.abs(ref).max())
    pyr = cb.corr_pyramid_build(f1, f2, L=4)
    out = torch.full((1, 324, H, W), float("nan"), device=f1.device)
    cb.corr_sample(f1, pyr, cs[1], out=out)
    err = float(np.abs(out.cpu().numpy().astype(np.float64) - ref).max())
    out.fill_(float("nan"))
    cb.corr_sample(f1, pyr, cs[1], out=out, prec=cb.CORR_PREC_BF16)
    err16 = float(np.abs(out.cpu().numpy().astype(np.float64) - ref).max())
    b16 = bf16_bound(h1, h2, ref)
    print("width %d D %d map %dx%d: bf16x3 max|err| %.2e (bound %.2e), bf16 max|err| %.2e (bound %.2e)"
          % (width, D, H, W, err, FP32_TOL * maxc, err16, b16), flush=True)
    assert err <= FP32_TOL * maxc
    assert err16 <= b16
    pyr.destroy()

"""The seeded input generators: shapes, determinism, and the stated structure."""
import numpy as np

from paper_2505_16942_amd import synth


def test_configs_have_the_stated_shapes():
    want = {"tiny": (1, 46, 62), "1080p": (1, 135, 240), "4k": (1, 270, 480), "8k": (1, 540, 960),
            "voronoi": (2, 270, 480)}
    for name, (B, H, W) in want.items():
        c = synth.config(name)
        assert (c["B"], c["H"], c["W"], c["D"], c["L"], c["r"]) == (B, H, W, 256, 4, 4)
        assert c["seed"] == 1000 + c["index"]


def test_tiny_is_deterministic_and_in_range():
    cfg = synth.config("tiny")
    f1, f2 = synth.features(cfg)
    g1, g2 = synth.features(cfg)
    assert f1.shape == (1, 256, 46, 62) and f1.dtype == np.float32
    assert np.array_equal(f1, g1) and np.array_equal(f2, g2)
    c = synth.coords(cfg)
    ys, xs = np.meshgrid(np.arange(46), np.arange(62), indexing="ij")
    assert np.all(np.abs(c[0, 0] - xs) <= 8.0 + 1e-4) and np.all(np.abs(c[0, 1] - ys) <= 8.0 + 1e-4)
    assert abs(float(f1.std()) - 1.0) < 0.01


def test_smooth_field_amplitude_and_outliers():
    cfg = synth.config("8k")
    small = dict(cfg, H=54, W=96)
    c = synth.coords(small)
    ys, xs = np.meshgrid(np.arange(54), np.arange(96), indexing="ij")
    flow = np.stack([c[0, 0] - xs, c[0, 1] - ys])
    big = np.abs(flow).max(axis=0) > 96 + 4      # beyond smooth amplitude + jitter: the outliers
    assert 0.01 < big.mean() < 0.06
    assert np.abs(flow).max() <= 200.0 + 1e-3


def test_walk_accumulates_between_lookups():
    cfg = dict(synth.config("4k"), H=27, W=48)
    c0, c5 = synth.coords(cfg, 0), synth.coords(cfg, 5)
    d = (c5 - c0).astype(np.float64)
    assert 1.5 < d.std() < 3.0          # sqrt(5) ~ 2.24

"""Seeded synthetic inputs for the correlation-lookup path.

This module only *draws inputs* (feature maps and lookup coordinates). It holds
none of the method's arithmetic (no correlation, no pooling, no lookup) and is
the one piece shared by the CPU oracle's tests and the GPU path's tests/bench.

The paper's isolated benchmark (Sec. "Isolated Sampling Evaluation") uses random
feature vectors and query centroids taken from RAFT on Sintel at 1/8 resolution,
with D = 256, 4 pyramid levels, r = 4. Neither Sintel nor RAFT weights are
available here, so the coordinates are synthetic stand-ins with the same shapes
and a comparable structure (smooth motion + jitter + outliers / piecewise
constant motion). No dataset item is reproduced.

All generators are deterministic functions of (config name, seed).
"""
from __future__ import annotations

import numpy as np

# name -> parameters.  H, W are feature-map sizes (1/8 of the frame).
CONFIGS = {
    # configs[0]: tiny single pair, maximally incoherent small-range flow
    "tiny": dict(index=0, B=1, H=46, W=62, D=256, L=4, r=4, features="iid",
                 flow="uniform", flow_range=8.0, lookups=1),
    # configs[1]: 1080p-input pair
    "1080p": dict(index=1, B=1, H=135, W=240, D=256, L=4, r=4, features="warp",
                  flow="smooth", amplitude=24.0, jitter=0.5, lookups=1),
    # configs[2]: 4K-input pair, 12 successive lookups (recurrent pattern)
    "4k": dict(index=2, B=1, H=270, W=480, D=256, L=4, r=4, features="warp",
               flow="smooth", amplitude=48.0, jitter=0.5, lookups=12, walk=1.0),
    # configs[3]: 8K-input pair with 5% outliers
    "8k": dict(index=3, B=1, H=540, W=960, D=256, L=4, r=4, features="warp",
               flow="smooth", amplitude=96.0, jitter=0.5, lookups=1,
               outlier_frac=0.05, outlier_range=200.0),
    # configs[4]: batched, piecewise-constant motion over Voronoi regions
    "voronoi": dict(index=4, B=2, H=270, W=480, D=256, L=4, r=4, features="warp",
                    flow="voronoi", regions=16, region_range=150.0, jitter=1.0,
                    lookups=1),
}


def config(name: str) -> dict:
    c = dict(CONFIGS[name])
    c["name"] = name
    c["seed"] = 1000 + c["index"]
    return c


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, stream]))


def smooth_field(rng: np.random.Generator, H: int, W: int, amplitude: float) -> np.ndarray:
    """[2, H, W] float64: per axis a sum of 4 sinusoids with random phase,
    0.5..3 cycles per image in each direction, non-negative amplitudes summing
    to `amplitude` (so |F| <= amplitude everywhere)."""
    ys, xs = np.meshgrid(np.arange(H, dtype=np.float64), np.arange(W, dtype=np.float64), indexing="ij")
    out = np.zeros((2, H, W), dtype=np.float64)
    for axis in range(2):
        a = rng.random(4) + 0.05
        a = a / a.sum() * amplitude
        fx = rng.uniform(0.5, 3.0, 4)
        fy = rng.uniform(0.5, 3.0, 4)
        ph = rng.uniform(0.0, 2.0 * np.pi, 4)
        for k in range(4):
            out[axis] += a[k] * np.sin(2.0 * np.pi * (fx[k] * xs / W + fy[k] * ys / H) + ph[k])
    return out


def voronoi_field(rng: np.random.Generator, H: int, W: int, regions: int, rng_range: float) -> np.ndarray:
    """[2, H, W] float64: constant flow per nearest-seed region."""
    sy = rng.uniform(0, H, regions)
    sx = rng.uniform(0, W, regions)
    fl = rng.uniform(-rng_range, rng_range, (regions, 2))
    ys, xs = np.meshgrid(np.arange(H, dtype=np.float64), np.arange(W, dtype=np.float64), indexing="ij")
    d2 = (ys[None] - sy[:, None, None]) ** 2 + (xs[None] - sx[:, None, None]) ** 2
    owner = np.argmin(d2, axis=0)
    return np.stack([fl[owner, 0], fl[owner, 1]], axis=0)


def _base_flow(cfg: dict, b: int) -> np.ndarray:
    """The motion field of batch item b (drives both the warp of fmap2 and the
    lookups): [2, H, W] float64, channel 0 = x displacement, 1 = y."""
    H, W = cfg["H"], cfg["W"]
    rng = _rng(cfg["seed"], 10 + b)
    if cfg["flow"] == "smooth":
        return smooth_field(rng, H, W, cfg["amplitude"])
    if cfg["flow"] == "voronoi":
        return voronoi_field(rng, H, W, cfg["regions"], cfg["region_range"])
    if cfg["flow"] == "uniform":
        return rng.uniform(-cfg["flow_range"], cfg["flow_range"], (2, H, W))
    raise ValueError(cfg["flow"])


def _warp(f1: np.ndarray, flow: np.ndarray) -> np.ndarray:
    """f2(q) = f1 sampled at q - flow(q), linear interpolation, zero outside.
    f1: [D, H, W] float32 -> [D, H, W] float32.  Input synthesis only."""
    D, H, W = f1.shape
    ys, xs = np.meshgrid(np.arange(H, dtype=np.float64), np.arange(W, dtype=np.float64), indexing="ij")
    px = xs - flow[0]
    py = ys - flow[1]
    x0 = np.floor(px).astype(np.int64)
    y0 = np.floor(py).astype(np.int64)
    ax = (px - x0).astype(np.float32)
    ay = (py - y0).astype(np.float32)
    # gather whole feature vectors (rows of a channels-last copy)
    rows = np.ascontiguousarray(f1.reshape(D, H * W).T)
    acc = np.zeros((H * W, D), dtype=np.float32)
    for dy in (0, 1):
        for dx in (0, 1):
            xi = x0 + dx
            yi = y0 + dy
            ok = (xi >= 0) & (xi < W) & (yi >= 0) & (yi < H)
            wgt = ((ax if dx else 1.0 - ax) * (ay if dy else 1.0 - ay) * ok).astype(np.float32)
            idx = (np.clip(yi, 0, H - 1) * W + np.clip(xi, 0, W - 1)).reshape(-1)
            acc += rows[idx] * wgt.reshape(-1, 1)
    return np.ascontiguousarray(acc.T).reshape(D, H, W)


def features(cfg: dict) -> tuple[np.ndarray, np.ndarray]:
    """(fmap1, fmap2), each float32 [B, D, H, W] (dense NCHW)."""
    B, D, H, W = cfg["B"], cfg["D"], cfg["H"], cfg["W"]
    rng = _rng(cfg["seed"], 1)
    f1 = rng.standard_normal((B, D, H, W), dtype=np.float32)
    if cfg["features"] == "iid":
        f2 = _rng(cfg["seed"], 2).standard_normal((B, D, H, W), dtype=np.float32)
        return f1, f2
    f2 = np.empty_like(f1)
    nrng = _rng(cfg["seed"], 2)
    for b in range(B):
        flow = _base_flow(cfg, b)
        f2[b] = _warp(f1[b], flow)
        f2[b] += np.float32(0.1) * nrng.standard_normal((D, H, W), dtype=np.float32)
    return f1, f2


def coords(cfg: dict, lookup: int = 0) -> np.ndarray:
    """Lookup coordinates for lookup number `lookup` (0-based): float32
    [B, 2, H, W], channel 0 = x, 1 = y, absolute position in level-0 pixels of
    fmap2 (pixel grid + flow)."""
    B, H, W = cfg["B"], cfg["H"], cfg["W"]
    ys, xs = np.meshgrid(np.arange(H, dtype=np.float64), np.arange(W, dtype=np.float64), indexing="ij")
    out = np.empty((B, 2, H, W), dtype=np.float32)
    for b in range(B):
        flow = _base_flow(cfg, b).copy()
        rng = _rng(cfg["seed"], 100 + b)
        if cfg.get("jitter", 0.0) > 0:
            flow += rng.normal(0.0, cfg["jitter"], (2, H, W))
        if cfg.get("outlier_frac", 0.0) > 0:
            mask = rng.random((H, W)) < cfg["outlier_frac"]
            rnd = rng.uniform(-cfg["outlier_range"], cfg["outlier_range"], (2, H, W))
            flow = np.where(mask[None], rnd, flow)
        # recurrent pattern: a per-pixel random walk of the flow between lookups
        walk = cfg.get("walk", 0.0)
        if walk > 0:
            for t in range(1, lookup + 1):
                flow += _rng(cfg["seed"], 1000 * t + b).normal(0.0, walk, (2, H, W))
        elif lookup > 0 and cfg.get("jitter", 0.0) > 0:
            # configs without a walk: a fresh jitter draw per lookup
            flow += _rng(cfg["seed"], 1000 * lookup + b).normal(0.0, cfg["jitter"], (2, H, W))
        out[b, 0] = (xs + flow[0]).astype(np.float32)
        out[b, 1] = (ys + flow[1]).astype(np.float32)
    return out


def small_case(seed: int, B: int, H: int, W: int, D: int, flow_range: float = 6.0,
               integer_coords: bool = False) -> tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Small iid case for tests: (fmap1, fmap2, coords)."""
    rng = _rng(seed, 7)
    f1 = rng.standard_normal((B, D, H, W), dtype=np.float32)
    f2 = rng.standard_normal((B, D, H, W), dtype=np.float32)
    ys, xs = np.meshgrid(np.arange(H, dtype=np.float64), np.arange(W, dtype=np.float64), indexing="ij")
    fl = rng.uniform(-flow_range, flow_range, (B, 2, H, W))
    if integer_coords:
        fl = np.round(fl)
    c = np.empty((B, 2, H, W), dtype=np.float32)
    c[:, 0] = xs[None] + fl[:, 0]
    c[:, 1] = ys[None] + fl[:, 1]
    return f1, f2, c

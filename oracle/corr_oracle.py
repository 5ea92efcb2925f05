"""ctypes front end of the CPU oracle (oracle/corr_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module
and this module never imports the product package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "corr_oracle.c")
_SRC_BACKWARD = os.path.join(_HERE, "corr_oracle_backward.c")
_LIB = os.path.join(_HERE, "libcorr_oracle.so")
_lib = None
# The mutation test loads deliberately broken builds of the oracle through this variable to show
# that the pins reject them; nothing else sets it.
_OVERRIDE = os.environ.get("CORR_ORACLE_LIB_OVERRIDE")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp64, OpenMP over queries)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_BACKWARD))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-ffp-contract=off", "-o", tmp, _SRC, _SRC_BACKWARD, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if _OVERRIDE:
            lib = ctypes.CDLL(_OVERRIDE)
        else:
            build()
            lib = ctypes.CDLL(_LIB)
        f32p = np.ctypeslib.ndpointer(np.float32, flags="C_CONTIGUOUS")
        f64p = np.ctypeslib.ndpointer(np.float64, flags="C_CONTIGUOUS")
        i64p = np.ctypeslib.ndpointer(np.int64, flags="C_CONTIGUOUS")
        ci = ctypes.c_int
        lib.corr_oracle_threads.restype = ci
        lib.corr_oracle_pyramid.argtypes = [f32p, ci, ci, ci, ci, ci, f64p]
        lib.corr_oracle_pyramid.restype = ci
        lib.corr_oracle_lookup.argtypes = [f32p, f32p, f32p, ci, ci, ci, ci, ci, ci, f64p]
        lib.corr_oracle_lookup.restype = ci
        lib.corr_oracle_lookup_points.argtypes = [f32p, f32p, f32p, ci, ci, ci, ci, ci, ci,
                                                  i64p, ctypes.c_long, f64p]
        lib.corr_oracle_lookup_points.restype = ci
        if hasattr(lib, "corr_oracle_backward"):          # absent from the mutation test's single-file builds
            lib.corr_oracle_backward.argtypes = [f32p, f32p, f32p, f64p, ci, ci, ci, ci, ci, ci, f64p, f64p]
            lib.corr_oracle_backward.restype = ci
        _lib = lib
    return _lib


def threads() -> int:
    return int(_load().corr_oracle_threads())


def level_sizes(H: int, W: int, L: int):
    out = []
    for _ in range(L):
        out.append((H, W))
        H, W = H // 2, W // 2
    return out


def _prep(fmap1, fmap2, coords):
    f1 = np.ascontiguousarray(fmap1, dtype=np.float32)
    f2 = np.ascontiguousarray(fmap2, dtype=np.float32)
    c = np.ascontiguousarray(coords, dtype=np.float32)
    B, D, H, W = f1.shape
    assert f2.shape == f1.shape, "equal-size feature maps"
    assert c.shape == (B, 2, H, W)
    return f1, f2, c, B, D, H, W


def pyramid(fmap2, L: int):
    """List of pooled target features, fp64 [B, D, H_l, W_l] per level."""
    f2 = np.ascontiguousarray(fmap2, dtype=np.float32)
    B, D, H, W = f2.shape
    sizes = level_sizes(H, W, L)
    total = sum(B * D * h * w for h, w in sizes)
    buf = np.empty(total, dtype=np.float64)
    rc = _load().corr_oracle_pyramid(f2, B, D, H, W, L, buf)
    if rc:
        raise RuntimeError("corr_oracle_pyramid failed: %d" % rc)
    out, off = [], 0
    for h, w in sizes:
        n = B * D * h * w
        out.append(buf[off:off + n].reshape(B, D, h, w))
        off += n
    return out


def lookup(fmap1, fmap2, coords, L: int = 4, r: int = 4) -> np.ndarray:
    """Full lookup: fp64 [B, L*(2r+1)^2, H, W]."""
    f1, f2, c, B, D, H, W = _prep(fmap1, fmap2, coords)
    K = 2 * r + 1
    out = np.empty((B, L * K * K, H, W), dtype=np.float64)
    rc = _load().corr_oracle_lookup(f1, f2, c, B, H, W, D, L, r, out)
    if rc:
        raise RuntimeError("corr_oracle_lookup failed: %d" % rc)
    return out


def lookup_points(fmap1, fmap2, coords, flat_idx, L: int = 4, r: int = 4) -> np.ndarray:
    """Selected outputs: flat indices into [B, L*(2r+1)^2, H, W] -> fp64 values."""
    f1, f2, c, B, D, H, W = _prep(fmap1, fmap2, coords)
    idx = np.ascontiguousarray(flat_idx, dtype=np.int64)
    vals = np.empty(idx.shape[0], dtype=np.float64)
    rc = _load().corr_oracle_lookup_points(f1, f2, c, B, H, W, D, L, r, idx, idx.shape[0], vals)
    if rc:
        raise RuntimeError("corr_oracle_lookup_points failed: %d" % rc)
    return vals


def backward(fmap1, fmap2, coords, d_out, L: int = 4, r: int = 4):
    """Gradients of sum(d_out * lookup) with respect to fmap1 and fmap2 (coordinates are constants):
    two fp64 arrays [B, D, H, W]."""
    f1, f2, c, B, D, H, W = _prep(fmap1, fmap2, coords)
    K = 2 * r + 1
    g = np.ascontiguousarray(d_out, dtype=np.float64)
    assert g.shape == (B, L * K * K, H, W)
    d1 = np.empty((B, D, H, W), dtype=np.float64)
    d2 = np.empty((B, D, H, W), dtype=np.float64)
    rc = _load().corr_oracle_backward(f1, f2, c, g, B, H, W, D, L, r, d1, d2)
    if rc:
        raise RuntimeError("corr_oracle_backward failed: %d" % rc)
    return d1, d2

"""Thin Python binding of the C-ABI library (include/corr.h).

Argument marshalling only: every step of the lookup runs in the library's HIP
kernels.  PyTorch supplies device memory and the current stream.  There is no
CPU fallback: if the library is missing or no GPU is visible, calls raise.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libcorr_mi355x.so")

CORR_OK = 0
CORR_ERR_INVALID_ARG, CORR_ERR_UNSUPPORTED, CORR_ERR_OOM, CORR_ERR_HIP, CORR_ERR_MISSING_REP = -1, -2, -3, -4, -5
CORR_MODE_BLOCK, CORR_MODE_ONDEMAND, CORR_MODE_FULLVOLUME = 0, 1, 2
CORR_PREC_BF16X3, CORR_PREC_BF16 = 0, 1
CORR_OUT_NCHW, CORR_OUT_NHWC = 0, 1
CORR_REP_SPLIT, CORR_REP_F32, CORR_REP_BF16 = 1, 2, 4

EXPORTS = [
    "corr_pyramid_build", "corr_pyramid_build_reps", "corr_pyramid_destroy", "corr_pyramid_bytes",
    "corr_sample", "corr_sample_mode", "corr_sample_layout", "corr_full_volume_bytes", "corr_workspace_bytes",
    "corr_last_block_stats", "corr_profile_enable", "corr_profile_read", "corr_bin_geometry",
    "corr_copy_f32", "corr_status_string",
]


class CorrError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__("%s: %s (%d)" % (what, status_string(status), status))


class BlockStats(ctypes.Structure):
    _fields_ = [("items", ctypes.c_int64), ("query_levels", ctypes.c_int64),
                ("null_query_levels", ctypes.c_int64), ("mma_point_queries", ctypes.c_int64),
                ("used_point_queries", ctypes.c_int64),
                ("level_items", ctypes.c_int64 * 4), ("level_mma_point_queries", ctypes.c_int64 * 4),
                ("level_used_point_queries", ctypes.c_int64 * 4), ("level_queries", ctypes.c_int64 * 4)]


class Profile(ctypes.Structure):
    _fields_ = [("lookups", ctypes.c_int64), ("binning_ms", ctypes.c_double), ("block_ms", ctypes.c_double)]


_lib = None


def load_library():
    """dlopen the in-tree library and declare its signatures.  Fails loudly."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("%s is missing: run __graft_entry__.build() (hipcc) first" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci, cu, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_uint, ctypes.c_size_t
    lib.corr_pyramid_build.argtypes = [vp, vp, ci, ci, ci, ci, ci, ctypes.POINTER(vp), vp]
    lib.corr_pyramid_build.restype = ci
    lib.corr_pyramid_build_reps.argtypes = [vp, vp, ci, ci, ci, ci, ci, cu, ctypes.POINTER(vp), vp]
    lib.corr_pyramid_build_reps.restype = ci
    lib.corr_pyramid_destroy.argtypes = [vp]
    lib.corr_pyramid_destroy.restype = ci
    lib.corr_pyramid_bytes.argtypes = [vp]
    lib.corr_pyramid_bytes.restype = sz
    lib.corr_sample.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, vp]
    lib.corr_sample.restype = ci
    lib.corr_sample_mode.argtypes = [ci, ci, vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, vp]
    lib.corr_sample_mode.restype = ci
    lib.corr_sample_layout.argtypes = [ci, ci, ci, vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, vp]
    lib.corr_sample_layout.restype = ci
    lib.corr_full_volume_bytes.argtypes = [ci, ci, ci, ci]
    lib.corr_full_volume_bytes.restype = sz
    lib.corr_workspace_bytes.argtypes = [cu, ci, ci, ci, ci, ci]
    lib.corr_workspace_bytes.restype = sz
    lib.corr_last_block_stats.argtypes = [vp, ctypes.POINTER(BlockStats), vp]
    lib.corr_last_block_stats.restype = ci
    lib.corr_profile_enable.argtypes = [vp, ci]
    lib.corr_profile_enable.restype = ci
    lib.corr_profile_read.argtypes = [vp, ctypes.POINTER(Profile)]
    lib.corr_profile_read.restype = ci
    lib.corr_bin_geometry.argtypes = [ci, ci, ci, ci] + [ctypes.POINTER(ci)] * 6
    lib.corr_bin_geometry.restype = ci
    lib.corr_copy_f32.argtypes = [vp, vp, sz, vp]
    lib.corr_copy_f32.restype = ci
    lib.corr_status_string.argtypes = [ci]
    lib.corr_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().corr_status_string(int(status)).decode()


def corr_full_volume_bytes(B: int, H: int, W: int, L: int) -> int:
    return int(load_library().corr_full_volume_bytes(B, H, W, L))


def corr_workspace_bytes(reps: int, B: int, H: int, W: int, D: int, L: int) -> int:
    return int(load_library().corr_workspace_bytes(reps, B, H, W, D, L))


def corr_bin_geometry(H: int, W: int, L: int, l: int):
    vals = [ctypes.c_int() for _ in range(6)]
    st = load_library().corr_bin_geometry(H, W, L, l, *[ctypes.byref(v) for v in vals])
    if st != CORR_OK:
        raise CorrError(st, "corr_bin_geometry")
    return tuple(v.value for v in vals)   # cell_x, cell_y, window_x, window_y, cells_x, cells_y


def _dev_f32(t: torch.Tensor, name: str) -> int:
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise TypeError("%s must be a contiguous float32 tensor on the GPU" % name)
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class Pyramid:
    """Owner of a library pyramid handle."""

    def __init__(self, handle: int, B, H, W, D, L, reps):
        self.handle = ctypes.c_void_p(handle)
        self.B, self.H, self.W, self.D, self.L, self.reps = B, H, W, D, L, reps

    def bytes(self) -> int:
        return int(load_library().corr_pyramid_bytes(self.handle))

    def destroy(self):
        if self.handle is not None and self.handle.value:
            load_library().corr_pyramid_destroy(self.handle)
        self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def corr_pyramid_build(fmap1: torch.Tensor, fmap2: torch.Tensor, L: int = 4,
                       reps: int = CORR_REP_SPLIT, pyramid: Pyramid | None = None) -> Pyramid:
    """fmap1, fmap2: [B, D, H, W] fp32 on the GPU.  Reuses `pyramid` if given."""
    lib = load_library()
    p1, p2 = _dev_f32(fmap1, "fmap1"), _dev_f32(fmap2, "fmap2")
    if fmap1.dim() != 4 or fmap1.shape != fmap2.shape:
        raise ValueError("fmap1 and fmap2 must both be [B, D, H, W]")
    B, D, H, W = (int(v) for v in fmap1.shape)
    handle = ctypes.c_void_p(pyramid.handle.value if pyramid is not None else None)
    st = lib.corr_pyramid_build_reps(p1, p2, B, H, W, D, L, reps, ctypes.byref(handle), _stream())
    if st != CORR_OK:
        raise CorrError(st, "corr_pyramid_build")
    if pyramid is not None:
        return pyramid
    return Pyramid(handle.value, B, H, W, D, L, reps)


def corr_sample(fmap1, pyramid: Pyramid, coords: torch.Tensor, r: int = 4,
                out: torch.Tensor | None = None, mode: int = CORR_MODE_BLOCK,
                prec: int = CORR_PREC_BF16X3, layout: int = CORR_OUT_NCHW) -> torch.Tensor:
    """coords: [B, 2, H, W] fp32 on the GPU.  Returns out fp32: [B, L*(2r+1)^2, H, W] for
    CORR_OUT_NCHW, [B, H, W, L*(2r+1)^2] for CORR_OUT_NHWC."""
    lib = load_library()
    pc = _dev_f32(coords, "coords")
    B, H, W, D, L = pyramid.B, pyramid.H, pyramid.W, pyramid.D, pyramid.L
    if tuple(coords.shape) != (B, 2, H, W):
        raise ValueError("coords must be [B, 2, H, W] = %s" % ((B, 2, H, W),))
    K = 2 * r + 1
    shape = (B, H, W, L * K * K) if layout == CORR_OUT_NHWC else (B, L * K * K, H, W)
    if out is None:
        out = torch.empty(shape, dtype=torch.float32, device=coords.device)
    elif tuple(out.shape) != shape:
        raise ValueError("out has the wrong shape")
    po = _dev_f32(out, "out")
    p1 = fmap1.data_ptr() if isinstance(fmap1, torch.Tensor) else None
    st = lib.corr_sample_layout(mode, prec, layout, p1, pyramid.handle, pc, B, H, W, D, L, r, po, _stream())
    if st != CORR_OK:
        raise CorrError(st, "corr_sample")
    return out


def corr_last_block_stats(pyramid: Pyramid) -> dict:
    s = BlockStats()
    st = load_library().corr_last_block_stats(pyramid.handle, ctypes.byref(s), _stream())
    if st != CORR_OK:
        raise CorrError(st, "corr_last_block_stats")
    out = {}
    for k, ty in BlockStats._fields_:
        v = getattr(s, k)
        out[k] = int(v) if ty is ctypes.c_int64 else [int(x) for x in v]
    return out


def corr_copy_f32(dst: torch.Tensor, src: torch.Tensor) -> None:
    """Plain device copy through the library's copy kernel (counter calibration)."""
    pd, ps = _dev_f32(dst, "dst"), _dev_f32(src, "src")
    if dst.numel() != src.numel():
        raise ValueError("dst and src must have the same number of elements")
    st = load_library().corr_copy_f32(pd, ps, src.numel(), _stream())
    if st != CORR_OK:
        raise CorrError(st, "corr_copy_f32")


def corr_profile_enable(pyramid: Pyramid, enable: bool = True) -> None:
    st = load_library().corr_profile_enable(pyramid.handle, 1 if enable else 0)
    if st != CORR_OK:
        raise CorrError(st, "corr_profile_enable")


def corr_profile_read(pyramid: Pyramid) -> dict:
    p = Profile()
    st = load_library().corr_profile_read(pyramid.handle, ctypes.byref(p))
    if st != CORR_OK:
        raise CorrError(st, "corr_profile_read")
    return {"lookups": int(p.lookups), "binning_ms": float(p.binning_ms), "block_ms": float(p.block_ms)}

"""Thin Python binding of the C-ABI library (include/corr.h, include/corr_bench.h).

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
CORR_ERR_TOO_LARGE = -6
CORR_STATIC_SCRATCH_BYTES = 2 << 20
CORR_MODE_BLOCK, CORR_MODE_ONDEMAND, CORR_MODE_FULLVOLUME = 0, 1, 2
CORR_PREC_BF16X3, CORR_PREC_BF16 = 0, 1
CORR_OUT_NCHW, CORR_OUT_NHWC = 0, 1
CORR_REP_SPLIT, CORR_REP_F32, CORR_REP_BF16 = 1, 2, 4

# the method's boundary (include/corr.h)
EXPORTS = [
    "corr_pyramid_build", "corr_pyramid_build_reps", "corr_pyramid_destroy", "corr_pyramid_bytes",
    "corr_sample", "corr_sample_mode", "corr_sample_layout", "corr_sample_static",
    "corr_full_volume_bytes", "corr_workspace_bytes", "corr_status_string",
    "corr_backward_workspace_bytes", "corr_sample_backward",
]
# measurement and test hooks (include/corr_bench.h)
BENCH_EXPORTS = [
    "corr_last_block_stats", "corr_profile_enable", "corr_profile_read", "corr_bin_geometry", "corr_copy_f32",
    "corr_debug_read_plan", "corr_debug_cell_coords", "corr_debug_read_level", "corr_debug_item_map",
    "corr_debug_set_level_split",
    "corr_debug_set_backward_form",
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
    _fields_ = [("lookups", ctypes.c_int64), ("dropped", ctypes.c_int64),
                ("binning_ms", ctypes.c_double), ("block_ms", ctypes.c_double)]


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
    lib.corr_pyramid_destroy.argtypes = [vp, vp]
    lib.corr_pyramid_destroy.restype = ci
    lib.corr_pyramid_bytes.argtypes = [vp]
    lib.corr_pyramid_bytes.restype = sz
    lib.corr_sample.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, vp]
    lib.corr_sample.restype = ci
    lib.corr_sample_mode.argtypes = [ci, ci, vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, vp]
    lib.corr_sample_mode.restype = ci
    lib.corr_sample_layout.argtypes = [ci, ci, ci, vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, vp]
    lib.corr_sample_layout.restype = ci
    lib.corr_sample_static.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, vp]
    lib.corr_sample_static.restype = ci
    lib.corr_backward_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
    lib.corr_backward_workspace_bytes.restype = sz
    lib.corr_sample_backward.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, vp, vp, sz, vp]
    lib.corr_sample_backward.restype = ci
    lib.corr_full_volume_bytes.argtypes = [ci, ci, ci, ci]
    lib.corr_full_volume_bytes.restype = sz
    lib.corr_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, ci, ci]
    lib.corr_workspace_bytes.restype = sz
    lib.corr_last_block_stats.argtypes = [vp, ci, ctypes.POINTER(BlockStats), vp]
    lib.corr_last_block_stats.restype = ci
    lib.corr_profile_enable.argtypes = [ci]
    lib.corr_profile_enable.restype = ci
    lib.corr_profile_read.argtypes = [ctypes.POINTER(Profile)]
    lib.corr_profile_read.restype = ci
    lib.corr_bin_geometry.argtypes = [ci, ci, ci, ci] + [ctypes.POINTER(ci)] * 6
    lib.corr_bin_geometry.restype = ci
    lib.corr_copy_f32.argtypes = [vp, vp, sz, vp]
    lib.corr_copy_f32.restype = ci
    i32p = ctypes.POINTER(ctypes.c_int32)
    lib.corr_debug_read_plan.argtypes = [vp, i32p, i32p, sz, i32p, sz, vp]
    lib.corr_debug_read_plan.restype = ci
    lib.corr_debug_cell_coords.argtypes = [vp, ci] + [ctypes.POINTER(ci)] * 3
    lib.corr_debug_cell_coords.restype = ci
    lib.corr_debug_item_map.argtypes = [ci, ctypes.POINTER(ctypes.c_int32), ctypes.c_size_t, ctypes.POINTER(ci)]
    lib.corr_debug_item_map.restype = ci
    lib.corr_debug_set_level_split.argtypes = [ci]
    lib.corr_debug_set_level_split.restype = ci
    lib.corr_debug_set_backward_form.argtypes = [ci]
    lib.corr_debug_set_backward_form.restype = ci
    lib.corr_debug_read_level.argtypes = [vp, cu, ci, ctypes.POINTER(ctypes.c_float), vp]
    lib.corr_debug_read_level.restype = ci
    lib.corr_status_string.argtypes = [ci]
    lib.corr_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().corr_status_string(int(status)).decode()


def corr_full_volume_bytes(B: int, H: int, W: int, L: int) -> int:
    return int(load_library().corr_full_volume_bytes(B, H, W, L))


def corr_workspace_bytes(mode: int, B: int, H: int, W: int, D: int, L: int, r: int = 4) -> int:
    return int(load_library().corr_workspace_bytes(mode, B, H, W, D, L, r))


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


def _stream_or_null():
    try:
        return torch.cuda.current_stream().cuda_stream
    except Exception:      # interpreter shutdown
        return None


class Pyramid:
    """Owner of a library pyramid handle."""

    def __init__(self, handle: int, B, H, W, D, L, reps):
        self.handle = ctypes.c_void_p(handle)
        self.B, self.H, self.W, self.D, self.L, self.reps = B, H, W, D, L, reps

    def bytes(self) -> int:
        return int(load_library().corr_pyramid_bytes(self.handle))

    def destroy(self):
        if self.handle is not None and self.handle.value:
            load_library().corr_pyramid_destroy(self.handle, _stream_or_null())
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


def corr_sample_static(fmap1, pyramid: Pyramid, coords: torch.Tensor, r: int = 4,
                       out: torch.Tensor | None = None) -> torch.Tensor:
    """corr_sample (block mode, bf16x3, NCHW) on the library's fixed planning scratch: allocates nothing
    inside the library.  Raises CorrError(CORR_ERR_TOO_LARGE) beyond the scratch size."""
    lib = load_library()
    pc = _dev_f32(coords, "coords")
    B, H, W, D, L = pyramid.B, pyramid.H, pyramid.W, pyramid.D, pyramid.L
    if tuple(coords.shape) != (B, 2, H, W):
        raise ValueError("coords must be [B, 2, H, W] = %s" % ((B, 2, H, W),))
    K = 2 * r + 1
    shape = (B, L * K * K, H, W)
    if out is None:
        out = torch.empty(shape, dtype=torch.float32, device=coords.device)
    elif tuple(out.shape) != shape:
        raise ValueError("out has the wrong shape")
    po = _dev_f32(out, "out")
    p1 = fmap1.data_ptr() if isinstance(fmap1, torch.Tensor) else None
    st = lib.corr_sample_static(p1, pyramid.handle, pc, B, H, W, D, L, r, po, _stream())
    if st != CORR_OK:
        raise CorrError(st, "corr_sample_static")
    return out


def corr_backward_workspace_bytes(B: int, H: int, W: int, D: int, L: int) -> int:
    return int(load_library().corr_backward_workspace_bytes(B, H, W, D, L))


def corr_sample_backward(pyramid: Pyramid, coords: torch.Tensor, d_out: torch.Tensor, r: int = 4,
                         d_fmap1: torch.Tensor | None = None, d_fmap2: torch.Tensor | None = None,
                         workspace: torch.Tensor | None = None):
    """Gradients of sum(d_out * lookup) with respect to fmap1 and fmap2: two fp32 tensors [B, D, H, W].
    `workspace`: a device buffer of at least corr_backward_workspace_bytes() bytes (allocated here if None)."""
    lib = load_library()
    pc = _dev_f32(coords, "coords")
    pg = _dev_f32(d_out, "d_out")
    B, H, W, D, L = pyramid.B, pyramid.H, pyramid.W, pyramid.D, pyramid.L
    K = 2 * r + 1
    if tuple(coords.shape) != (B, 2, H, W):
        raise ValueError("coords must be [B, 2, H, W] = %s" % ((B, 2, H, W),))
    if tuple(d_out.shape) != (B, L * K * K, H, W):
        raise ValueError("d_out must be [B, L*K*K, H, W] = %s" % ((B, L * K * K, H, W),))
    need = corr_backward_workspace_bytes(B, H, W, D, L)
    if workspace is None:
        workspace = torch.empty(need // 4, dtype=torch.float32, device=coords.device)
    if workspace.device != coords.device or not workspace.is_contiguous() or workspace.numel() * workspace.element_size() < need:
        raise ValueError("workspace must be a contiguous device buffer of at least %d bytes" % need)
    outs = []
    for t, name in ((d_fmap1, "d_fmap1"), (d_fmap2, "d_fmap2")):
        if t is None:
            t = torch.empty((B, D, H, W), dtype=torch.float32, device=coords.device)
        elif tuple(t.shape) != (B, D, H, W):
            raise ValueError("%s must be [B, D, H, W]" % name)
        _dev_f32(t, name)
        outs.append(t)
    st = lib.corr_sample_backward(pyramid.handle, pc, pg, B, H, W, D, L, r, outs[0].data_ptr(), outs[1].data_ptr(),
                                  workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream())
    if st != CORR_OK:
        raise CorrError(st, "corr_sample_backward")
    return outs[0], outs[1]


def corr_last_block_stats(pyramid: Pyramid, r: int = 4) -> dict:
    s = BlockStats()
    st = load_library().corr_last_block_stats(pyramid.handle, r, ctypes.byref(s), _stream())
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


def corr_profile_enable(enable: bool = True) -> None:
    st = load_library().corr_profile_enable(1 if enable else 0)
    if st != CORR_OK:
        raise CorrError(st, "corr_profile_enable")


def corr_profile_read() -> dict:
    p = Profile()
    st = load_library().corr_profile_read(ctypes.byref(p))
    if st != CORR_OK:
        raise CorrError(st, "corr_profile_read")
    return {"lookups": int(p.lookups), "dropped": int(p.dropped),
            "binning_ms": float(p.binning_ms), "block_ms": float(p.block_ms)}


def corr_debug_read_plan(pyramid: Pyramid):
    """(items [n, 4] int32, perm [m] int32) of the last block-mode lookup on this pyramid."""
    import numpy as np
    BN = pyramid.B * pyramid.H * pyramid.W
    counts = np.zeros(2, np.int32)
    items = np.zeros((BN + 65536, 4), np.int32)
    perm = np.zeros(BN, np.int32)
    i32p = ctypes.POINTER(ctypes.c_int32)
    st = load_library().corr_debug_read_plan(pyramid.handle, counts.ctypes.data_as(i32p), items.ctypes.data_as(i32p),
                                             items.shape[0], perm.ctypes.data_as(i32p), perm.size, _stream())
    if st != CORR_OK:
        raise CorrError(st, "corr_debug_read_plan")
    return items[:counts[0]].copy(), perm[:counts[1]].copy()


CORR_BACKWARD_ITEMS, CORR_BACKWARD_QUERIES = 0, 1


def corr_debug_set_backward_form(form: int) -> int:
    """Which kernel corr_sample_backward runs (CORR_BACKWARD_ITEMS, the default, or CORR_BACKWARD_QUERIES);
    returns the previous setting."""
    return int(load_library().corr_debug_set_backward_form(int(form)))


def corr_debug_set_level_split(max_queries: int) -> int:
    """Block mode on inputs of up to `max_queries` queries is launched with the kernel that can run an item's
    levels in workgroups of their own; 0 = never, -1 = the default, -2 / -4 = always two / four ways.
    Returns the previous setting."""
    return int(load_library().corr_debug_set_level_split(int(max_queries)))


def corr_debug_item_map(max_items: int):
    """(grid, map): the block kernel's grid for `max_items` and the item index each workgroup takes."""
    import numpy as np
    lib = load_library()
    grid = ctypes.c_int()
    st = lib.corr_debug_item_map(int(max_items), None, 0, ctypes.byref(grid))
    if st != CORR_OK:
        raise CorrError(st, "corr_debug_item_map")
    m = np.zeros(grid.value, np.int32)
    st = lib.corr_debug_item_map(int(max_items), m.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), m.size, ctypes.byref(grid))
    if st != CORR_OK:
        raise CorrError(st, "corr_debug_item_map")
    return grid.value, m


def corr_debug_cell_coords(pyramid: Pyramid, cell_id: int):
    vals = [ctypes.c_int() for _ in range(3)]
    st = load_library().corr_debug_cell_coords(pyramid.handle, int(cell_id), *[ctypes.byref(v) for v in vals])
    if st != CORR_OK:
        raise CorrError(st, "corr_debug_cell_coords")
    return tuple(v.value for v in vals)    # b, u, v


def corr_debug_read_level(pyramid: Pyramid, rep: int, level: int):
    """Level `level` of fmap2 (-1: fmap1) as the pyramid holds it: fp32 [B, H_l, W_l, D] numpy array."""
    import numpy as np
    Hl, Wl = (pyramid.H, pyramid.W) if level < 0 else (pyramid.H >> level, pyramid.W >> level)
    dst = np.zeros((pyramid.B, Hl, Wl, pyramid.D), np.float32)
    st = load_library().corr_debug_read_level(pyramid.handle, rep, level,
                                              dst.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), _stream())
    if st != CORR_OK:
        raise CorrError(st, "corr_debug_read_level")
    return dst

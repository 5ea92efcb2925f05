"""The C-ABI library loads and exports every symbol include/corr.h and include/corr_bench.h
declare; host-only entry points behave as documented.  No device work here."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "corr.h")
BENCH_HEADER = os.path.join(ROOT, "include", "corr_bench.h")


def _declared_functions(header=HEADER):
    src = open(header).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = re.findall(r"\b(corr_[a-z0-9_]+)\s*\(", src)
    return sorted(set(names))


def _lib():
    from paper_2505_16942_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        pytest.skip("library not built (run __graft_entry__.build())")
    return binding, ctypes.CDLL(binding.LIB_PATH)


def test_header_symbols_are_exported():
    binding, lib = _lib()
    declared = _declared_functions()
    assert "corr_pyramid_build" in declared and "corr_sample" in declared
    for name in declared:
        assert hasattr(lib, name), "missing export: " + name
    assert sorted(binding.EXPORTS) == declared
    hooks = _declared_functions(BENCH_HEADER)
    assert "corr_copy_f32" in hooks and not set(hooks) & set(declared)
    for name in hooks:
        assert hasattr(lib, name), "missing export: " + name
    assert sorted(binding.BENCH_EXPORTS) == hooks


def test_full_volume_bytes_matches_closed_form():
    binding, _ = _lib()
    # 4 * B * N * sum_l N_l with floor-halved levels
    for (B, H, W, L) in [(1, 46, 62, 4), (1, 135, 240, 4), (2, 270, 480, 4), (1, 540, 960, 4), (3, 17, 9, 2)]:
        n = sum((H >> l) * (W >> l) for l in range(L))
        assert binding.corr_full_volume_bytes(B, H, W, L) == 4 * B * H * W * n
    assert binding.corr_full_volume_bytes(1, 540, 960, 4) == 1427549184000
    assert binding.corr_full_volume_bytes(1, 4, 4, 4) == 0        # level 3 would be empty
    assert binding.corr_full_volume_bytes(0, 4, 4, 1) == 0


def test_status_strings_and_workspace():
    binding, _ = _lib()
    seen = {binding.status_string(s) for s in (0, -1, -2, -3, -4, -5, -6)}
    assert len(seen) == 7 and "ok" in seen
    feat = 4 * 256 * (540 * 960 + sum((540 >> l) * (960 >> l) for l in range(4)))
    ws = binding.corr_workspace_bytes(binding.CORR_MODE_BLOCK, 1, 540, 960, 256, 4, 4)
    assert feat < ws < feat * 1.02          # workspace beyond the features is linear in pixels and small (Eq. 4)
    assert binding.corr_workspace_bytes(binding.CORR_MODE_ONDEMAND, 1, 540, 960, 256, 4, 4) == feat
    assert binding.corr_workspace_bytes(binding.CORR_MODE_FULLVOLUME, 1, 540, 960, 256, 4, 4) == feat + 1427549184000
    # linear in the number of pixels: four times the pixels, about four times the bytes
    small = binding.corr_workspace_bytes(binding.CORR_MODE_BLOCK, 1, 270, 480, 256, 4, 4)
    assert 3.9 < ws / small < 4.1
    assert binding.corr_workspace_bytes(binding.CORR_MODE_BLOCK, 1, 16, 16, 48, 2, 4) == 0   # unsupported D
    assert binding.corr_workspace_bytes(binding.CORR_MODE_BLOCK, 1, 16, 16, 64, 2, 5) == 0   # unsupported r


def test_bin_geometry_matches_the_rule():
    binding, _ = _lib()
    for (H, W, L) in [(540, 960, 4), (46, 62, 4), (16, 24, 2), (9, 9, 1)]:
        for l in range(L):
            cx, cy, wx, wy, nx, ny = binding.corr_bin_geometry(H, W, L, l)
            assert cx == max(16 >> l, 1) and cy == max(8 >> l, 1)
            assert wx == cx + 9 and wy == cy + 9
            m = L - 1
            assert nx == ((((W >> m) + 4) * (1 << m) - 1) >> 4) - ((-5 * (1 << m)) >> 4) + 1
            assert ny == ((((H >> m) + 4) * (1 << m) - 1) >> 3) - ((-5 * (1 << m)) >> 3) + 1
    with pytest.raises(binding.CorrError):
        binding.corr_bin_geometry(4, 4, 4, 0)


def test_every_work_item_has_exactly_one_workgroup():
    """The block kernel's workgroup -> item mapping, enumerated on the host for every workspace size in a
    range and for the sizes of the benchmark configurations: a permutation of the launch grid, and the grid
    covers the largest item count the workspace can hold (an unvisited item would leave stale output)."""
    from paper_2505_16942_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        pytest.skip("library not built")
    sizes = list(range(0, 1200)) + [2047, 2048, 2049, 8191, 8192, 9713, 65535, 65537, 300001]
    for max_items in sizes:
        grid, m = binding.corr_debug_item_map(max_items)
        assert grid >= max_items and grid % 8 == 0
        assert np.array_equal(np.sort(m), np.arange(grid)), max_items
    # consecutive items stay on one XCD (workgroup w runs on XCD w % 8) in runs of 32 (one 4 x 8 super-tile of cells)
    grid, m = binding.corr_debug_item_map(4096)
    xcd_of_item = np.empty(grid, np.int64)
    xcd_of_item[m] = np.arange(grid) % 8
    assert np.all(xcd_of_item.reshape(-1, 32) == xcd_of_item.reshape(-1, 32)[:, :1])
    assert np.array_equal(xcd_of_item.reshape(-1, 32)[:8, 0], np.arange(8))


def test_backward_workspace_bytes():
    """Host arithmetic only: the gradient's workspace holds the channels-last gradient of fmap1 (one array per level
    up to 32000 queries, two up to 40000, one beyond), of every level of fmap2, and a planning workspace that is
    linear in pixels and small."""
    binding, _ = _lib()

    def grad_floats(B, H, W, D, L, parts):
        return (parts * B * H * W + B * sum((H >> l) * (W >> l) for l in range(L))) * D

    for (B, H, W, D, L, parts) in [(1, 30, 44, 64, 4, 4), (2, 100, 160, 256, 4, 4), (1, 135, 240, 256, 4, 2),
                                   (1, 135, 240, 256, 1, 1), (1, 270, 480, 256, 4, 1), (1, 540, 960, 256, 3, 1)]:
        need = binding.corr_backward_workspace_bytes(B, H, W, D, L)
        g = 4 * grad_floats(B, H, W, D, L, parts)
        plan = need - g
        assert need % 256 == 0
        assert 0 < plan < 256 + 64 * B * H * W + (1 << 20), (B, H, W, D, L, need, g)

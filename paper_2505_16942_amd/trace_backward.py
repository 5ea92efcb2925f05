"""Per-phase time split of the gradient's item kernel, from clock readings it sums up in a trace build.

A library built with -DCORR_TRACE (CORR_EXTRA_HIPCC_FLAGS=-DCORR_TRACE python -m paper_2505_16942_amd.build)
exports corr_debug_set_backward_trace; thread 0 of every work item then adds the 100 MHz wall clock up
per phase (set-up, staging a level's tap gradients, clearing G, the footprint scatter, the two
contractions, the final store), with a workgroup barrier in front of every reading.  This script runs one
corr_sample_backward of a benchmark configuration with tracing on and prints the mean time of each phase
per item, overall and by how many 16-query tiles the items fill.  The barriers and readings cost a few
percent; the plain build is what bench.py times.

Usage (GPU machine, repository root):  python -m paper_2505_16942_amd.trace_backward [4k] [--lib path/to/lib.so]
"""
from __future__ import annotations

import argparse
import ctypes
import sys

PHASES = ["set-up", "tap gradients to LDS", "clear G, row table", "footprint scatter", "d f1 contraction",
          "d f2 contraction + atomics", "store d f1"]


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("config", nargs="?", default="4k")
    ap.add_argument("--lib", default=None, help="trace build of the library (default: the in-tree library)")
    args = ap.parse_args(argv)
    import torch
    from . import binding as b
    from . import synth
    if args.lib:
        b.LIB_PATH = args.lib
    lib = b.load_library()
    if not hasattr(lib, "corr_debug_set_backward_trace"):
        print("trace_backward: this library was not built with -DCORR_TRACE", file=sys.stderr)
        return 1
    fn = lib.corr_debug_set_backward_trace
    fn.argtypes = [ctypes.c_void_p]
    fn.restype = None
    dev = torch.device("cuda:0")
    cfg = synth.config(args.config)
    f1, f2 = synth.features(cfg)
    t1, t2, tc = (torch.from_numpy(a).to(dev) for a in (f1, f2, synth.coords(cfg, 0)))
    B, D, H, W = t1.shape
    L, r = cfg["L"], cfg["r"]
    K = 2 * r + 1
    gen = torch.Generator(device=dev)
    gen.manual_seed(cfg["seed"])
    d_out = torch.randn((B, L * K * K, H, W), device=dev, generator=gen)
    pyr = b.corr_pyramid_build(t1, t2, L=L, reps=b.CORR_REP_F32)
    ws = torch.empty(b.corr_backward_workspace_bytes(B, H, W, D, L) // 4, device=dev)
    g1, g2 = torch.empty_like(t1), torch.empty_like(t1)
    b.corr_sample_backward(pyr, tc, d_out, r=r, d_fmap1=g1, d_fmap2=g2, workspace=ws)      # warm-up
    torch.cuda.synchronize()
    # one row per workgroup of the item kernel's grid (never more than one per query plus a few)
    tr = torch.zeros((B * H * W + B * H * W // 64 + 1024, 8), dtype=torch.int64, device=dev)
    fn(tr.data_ptr())
    b.corr_sample_backward(pyr, tc, d_out, r=r, d_fmap1=g1, d_fmap2=g2, workspace=ws)
    torch.cuda.synchronize()
    fn(None)
    t = tr.cpu().numpy()
    t = t[t[:, 7] > 0]
    us = t[:, :7] / 100.0
    total = us.sum(1).mean()
    print("%s: %d items, %.2f 16-query tiles per item on average, %.1f us per item" % (args.config, len(t), t[:, 7].mean(), total))
    print("| phase | us per item | share |")
    print("|---|---|---|")
    for i, name in enumerate(PHASES):
        print("| %s | %.1f | %.1f %% |" % (name, us[:, i].mean(), 100.0 * us[:, i].mean() / total))
    print()
    print("| tiles | items | " + " | ".join(PHASES) + " |")
    print("|---|---|" + "---|" * len(PHASES))
    for nm in range(1, 9):
        sel = us[t[:, 7] == nm]
        if len(sel):
            print("| %d | %d | " % (nm, len(sel)) + " | ".join("%.1f" % sel[:, i].mean() for i in range(7)) + " |")
    pyr.destroy()
    return 0


if __name__ == "__main__":
    sys.exit(main())

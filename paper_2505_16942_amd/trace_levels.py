"""Per-phase time split of the block kernel, from timestamps the kernel writes in a trace build.

A library built with -DCORR_TRACE (CORR_EXTRA_HIPCC_FLAGS=-DCORR_TRACE python -m paper_2505_16942_amd.build)
exports corr_debug_set_trace; thread 0 of every work item then stores the 100 MHz wall clock at the
start of the item, after its query fragments are in, and after every level's chunk loop and epilogue.
This script runs one lookup of a benchmark configuration with tracing on and prints the mean duration
of each phase, by how full the items are.  Timestamps cost a few percent; the plain build is what
bench.py times.

Usage (GPU machine, repository root):  python -m paper_2505_16942_amd.trace_levels [8k] [--lib path/to/lib.so]
"""
from __future__ import annotations

import argparse
import ctypes
import sys


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("config", nargs="?", default="8k")
    ap.add_argument("--lib", default=None, help="trace build of the library (default: the in-tree library)")
    args = ap.parse_args(argv)
    import numpy as np
    import torch
    from . import binding as b
    from . import synth
    if args.lib:
        b.LIB_PATH = args.lib
    lib = b.load_library()
    if not hasattr(lib, "corr_debug_set_trace"):
        print("trace_levels: this library was not built with -DCORR_TRACE", file=sys.stderr)
        return 1
    dev = torch.device("cuda:0")
    cfg = synth.config(args.config)
    f1, f2 = synth.features(cfg)
    t1, t2, tc = (torch.from_numpy(a).to(dev) for a in (f1, f2, synth.coords(cfg, 0)))
    pyr = b.corr_pyramid_build(t1, t2, L=cfg["L"])
    out = b.corr_sample(t1, pyr, tc)
    torch.cuda.synchronize()
    items, _ = b.corr_debug_read_plan(pyr)
    n = len(items)
    tr = torch.zeros((n + 512) * 16, dtype=torch.int64, device=dev)
    lib.corr_debug_set_trace.argtypes = [ctypes.c_void_p]
    lib.corr_debug_set_trace(tr.data_ptr())
    b.corr_profile_enable(True)
    b.corr_sample(t1, pyr, tc, out=out)
    torch.cuda.synchronize()
    prof = b.corr_profile_read()
    b.corr_profile_enable(False)
    lib.corr_debug_set_trace(None)
    t = tr.cpu().numpy().reshape(-1, 16)[:n].astype(np.float64)
    t[t == 0] = np.nan
    us = 0.01                                                # one tick of the 100 MHz clock
    d = np.diff(t[:, :10], axis=1) * us
    names = ["start (records, query fragments, first loads)"] + [x for l in range(4) for x in ("level %d chunk loop" % l, "level %d epilogue" % l)]
    nq = items[:, 2]
    groups = [("all items", nq > 0), ("1-64 queries", nq <= 64), ("65-128 queries", nq > 64)]
    print("block kernel, %s workload, trace build: %d work items, kernel %.3f ms" % (args.config, n, prof["block_ms"]))
    print("| phase | " + " | ".join("%s (%d), us" % (g, m.sum()) for g, m in groups) + " |")
    print("|---|" + "---|" * len(groups))
    for i, nm in enumerate(names):
        print("| %s | " % nm + " | ".join("%.2f" % np.nanmean(d[m, i]) for _, m in groups) + " |")
    print("| whole item | " + " | ".join("%.2f" % np.nanmean((t[m, 9] - t[m, 0]) * us) for _, m in groups) + " |")
    full = nq > 64
    tt = t[full]
    parts = (("plan next level + first loads", 2, 10), ("accumulators to LDS, round 0", 10, 11), ("taps, round 0", 11, 12),
             ("accumulators to LDS, round 1", 12, 13), ("taps, round 1", 13, 14))
    print("level 0 epilogue of items with more than 64 queries, us: " +
          ", ".join("%s %.2f" % (nm, np.nanmean(tt[:, e] - tt[:, s]) * us) for nm, s, e in parts))
    pyr.destroy()
    return 0


if __name__ == "__main__":
    sys.exit(main())

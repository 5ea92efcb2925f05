"""How often a per-query cache of enlarged footprints would serve the recurrent lookup pattern.

The cache this models: per query and level, the (10 + 2m)^2 correlation values around the integer
footprint origin floor(c / 2^l) - r of the lookup that filled it, m = margin in level-l pixels.  A later
lookup of the same query can be sampled from the cache at that level if its own origin lies within m
pixels of the cached one on both axes (hit); otherwise that query-level is recomputed and re-cached
(miss).  This script only counts: hit rates per level over the 12 lookups of a benchmark configuration
(host arithmetic on the seeded coordinates, no GPU), the cache size, and how the misses are spread
over the 16 x 8 target cells that the block kernel works by (a cell's window has to be loaded from
L2 if a single one of its queries misses).

Usage:  python -m paper_2505_16942_amd.reuse_model [4k]
"""
from __future__ import annotations

import sys

import numpy as np


def main(argv=None) -> int:
    from . import synth
    name = (argv or sys.argv[1:] or ["4k"])[0]
    cfg = synth.config(name)
    B, H, W, L = cfg["B"], cfg["H"], cfg["W"], cfg["L"]
    n = max(cfg.get("lookups", 1), 12)
    cs = [synth.coords(cfg, t).astype(np.float64) for t in range(n)]
    print("configuration %s: B=%d map %dx%d, %d lookups on one pyramid" % (name, B, H, W, n))
    print("| margin | level | hit rate, lookups 2..%d | cells with at least one miss | misses per such cell | cache bytes per query |" % n)
    print("|---|---|---|---|---|---|")
    for m in (1, 2, 3):
        for l in range(L):
            org = np.floor(cs[0] / 2 ** l)
            hits, cell_frac, per_cell = [], [], []
            for t in range(1, n):
                cur = np.floor(cs[t] / 2 ** l)
                hit = np.abs(cur - org).max(axis=1) <= m                   # [B, H, W]
                hits.append(hit.mean())
                cx = np.floor(cs[t][:, 0]).astype(np.int64) >> 4
                cy = np.floor(cs[t][:, 1]).astype(np.int64) >> 3
                key = (cy - cy.min()) * (cx.max() - cx.min() + 1) + (cx - cx.min())
                all_cells = np.unique(key).size
                miss_cells, counts = np.unique(key[~hit], return_counts=True)
                cell_frac.append(miss_cells.size / all_cells)
                per_cell.append(counts.mean() if counts.size else 0.0)
                org = np.where(hit[:, None], org, cur)                      # a miss refills the entry
            print("| %d | %d | %.3f | %.3f | %.1f | %d |" % (m, l, np.mean(hits), np.mean(cell_frac), np.mean(per_cell),
                                                              (10 + 2 * m) ** 2 * 4))
    return 0


if __name__ == "__main__":
    sys.exit(main())

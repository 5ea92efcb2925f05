"""Turns rocprofv3 CSV output of `bench.py` runs into the short text summaries kept under profiles/.

    python3 -m paper_2505_16942_amd.profile_summary stats   <dir of a --kernel-trace run>
    python3 -m paper_2505_16942_amd.profile_summary traffic <dir of the FETCH_SIZE run> <dir of the WRITE_SIZE run> --config 8k
    python3 -m paper_2505_16942_amd.profile_summary counters <dir of a --pmc run> [<dir> ...]

`stats` splits every kernel's launches by launch grid, so that the block kernel's 8k launches and 4k
launches (one bench run times both workloads) get rows of their own.  `traffic` scales FETCH_SIZE and
WRITE_SIZE (KiB per dispatch) by what the same counters read for the library's plain copy kernel on
1 GiB (`bench.py --copy-calibration`), and records the hash of the kernel sources it measured.
"""
from __future__ import annotations

import argparse
import collections
import csv
import datetime
import glob
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _find(d: str, suffix: str) -> str:
    hits = sorted(glob.glob(os.path.join(d, "**", "*" + suffix), recursive=True))
    if not hits:
        raise SystemExit("no *%s under %s" % (suffix, d))
    return hits[-1]


def _short(name: str) -> str:
    name = name.replace("(anonymous namespace)::", "")
    return name if len(name) <= 90 else name[:87] + "..."


def _counter_rows(d: str):
    """{kernel: {counter: [value per dispatch]}} (a dispatch's per-XCD/per-instance rows are summed)."""
    per = collections.defaultdict(float)
    order = []
    for r in csv.DictReader(open(_find(d, "counter_collection.csv"))):
        key = (r["Dispatch_Id"], r["Kernel_Name"], r["Counter_Name"])
        if key not in per:
            order.append(key)
        per[key] += float(r["Counter_Value"])
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for key in order:
        acc[key[1]][key[2]].append(per[key])
    return acc


def kernel_source_sha() -> str:
    import hashlib
    csrc = os.path.join(ROOT, "paper_2505_16942_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()


def algorithmic_bytes(config: str) -> int:
    """HBM bytes one block-mode lookup has to move: fmap1 and every pyramid pixel once as bf16 hi+lo
    (4 B per element), coordinates, the sorted query list, `out` once."""
    from . import synth
    c = synth.config(config)
    B, H, W, D, L, r = c["B"], c["H"], c["W"], c["D"], c["L"], c["r"]
    K = 2 * r + 1
    N = H * W
    npyr = sum((H >> l) * (W >> l) for l in range(L))
    return B * (N * D * 4 + npyr * D * 4 + N * 8 + N * 4 + N * L * K * K * 4)


def cmd_stats(args) -> int:
    rows = collections.defaultdict(list)
    for r in csv.DictReader(open(_find(args.dir, "kernel_trace.csv"))):
        grid = int(r["Grid_Size_X"]) if "Grid_Size_X" in r else int(r.get("Grid_Size", 0))
        rows[(r["Kernel_Name"], grid)].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    total = sum(sum(v) for v in rows.values())
    print("| kernel | grid (threads) | calls | mean us | min us | max us | total ms | share |")
    print("|---|---|---|---|---|---|---|---|")
    for (name, grid), v in sorted(rows.items(), key=lambda kv: -sum(kv[1])):
        if sum(v) / total < 0.002 and not any(w in name for w in ("corr", "block", "bin", "bwd", "fill_i32")):
            continue
        print("| %s | %d | %d | %.1f | %.1f | %.1f | %.3f | %.1f %% |" % (
            _short(name), grid, len(v), sum(v) / len(v), min(v), max(v), sum(v) / 1e3, 100.0 * sum(v) / total))
    return 0


def cmd_traffic(args) -> int:
    fetch, write = _counter_rows(args.fetch_dir), _counter_rows(args.write_dir)

    def pick(acc, what, counter):
        hits = [(k, v[counter]) for k, v in acc.items() if what in k and counter in v]
        if not hits:
            raise SystemExit("no %s rows with %s" % (what, counter))
        if what == "block_kernel":                      # the instantiation with the most launches
            hits.sort(key=lambda kv: -len(kv[1]))
        return hits[0]

    gib_kib = float(1 << 20)
    _, cf = pick(fetch, "copy_f32_kernel", "FETCH_SIZE")
    _, cw = pick(write, "copy_f32_kernel", "WRITE_SIZE")
    sf, sw = gib_kib / (sum(cf) / len(cf)), gib_kib / (sum(cw) / len(cw))
    kname, bf = pick(fetch, "block_kernel", "FETCH_SIZE")
    _, bw = pick(write, "block_kernel", "WRITE_SIZE")
    rd = sum(bf) / len(bf) * sf * 1024.0
    wr = sum(bw) / len(bw) * sw * 1024.0
    alg = algorithmic_bytes(args.config)
    cmd = ("cd /tmp && export TMPDIR=/tmp && rocprofv3 --pmc %s --kernel-trace --output-format csv -d <out> -o pmc -- "
           "python3 <repo>/bench.py --config %s --no-cpu-baseline --no-4k --steps 1 --warmup 0 --copy-calibration")
    print("HBM traffic of %s per launch, %s workload, from two rocprofv3 counter runs" % (_short(kname), args.config))
    print("commands (MI355X box; one counter per run):")
    print("  " + cmd % ("FETCH_SIZE", args.config))
    print("  " + cmd % ("WRITE_SIZE", args.config))
    print("  python3 -m paper_2505_16942_amd.profile_summary traffic <out of the first> <out of the second> --config %s" % args.config)
    print("calibration kernel: copy_f32_kernel, 1 GiB read + 1 GiB written per launch (%d launches)" % len(cf))
    print("  FETCH_SIZE reads %.4g KiB for 1 GiB read    -> scale factor %.3f" % (sum(cf) / len(cf), sf))
    print("  WRITE_SIZE reads %.4g KiB for 1 GiB written -> scale factor %.3f" % (sum(cw) / len(cw), sw))
    print("block kernel, mean over %d launches:" % len(bf))
    print("  FETCH_SIZE %.4g KiB x %.3f = %d bytes read" % (sum(bf) / len(bf), sf, rd))
    print("  WRITE_SIZE %.4g KiB x %.3f = %d bytes written" % (sum(bw) / len(bw), sw, wr))
    print("algorithmic bytes per launch: %d (fmap1 + pyramid once as bf16 hi+lo, coords, query list, out once)" % alg)
    print("traffic / algorithmic = %.2f" % ((rd + wr) / alg))
    print("date: %s" % datetime.date.today().isoformat())
    print("kernel_source_sha256: %s" % kernel_source_sha())
    print("traffic_bytes_per_launch: %d" % (rd + wr))
    return 0


def cmd_counters(args) -> int:
    print("| kernel | counter | dispatches | mean per dispatch |")
    print("|---|---|---|---|")
    for d in args.dirs:
        for k, v in _counter_rows(d).items():
            if not any(w in k for w in ("block_kernel", "bin_", "build_features", "copy_f32", "bwd_")):
                continue
            for cname, vals in sorted(v.items()):
                print("| %s | %s | %d | %.6g |" % (_short(k), cname, len(vals), sum(vals) / len(vals)))
    return 0


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    p = sub.add_parser("stats"); p.add_argument("dir"); p.set_defaults(fn=cmd_stats)
    p = sub.add_parser("traffic"); p.add_argument("fetch_dir"); p.add_argument("write_dir")
    p.add_argument("--config", default="8k"); p.set_defaults(fn=cmd_traffic)
    p = sub.add_parser("counters"); p.add_argument("dirs", nargs="+"); p.set_defaults(fn=cmd_counters)
    args = ap.parse_args(argv)
    return args.fn(args)


if __name__ == "__main__":
    sys.exit(main())

"""One-variable sweeps of the isolated sampling benchmark (paper: appendix table
"Full correlation volume sampling isolated benchmarking results depending on
one variable": input width, number of iterations, feature dimensionality).

For each point the three modes of the library run the whole job of one image
pair — preprocessing (pyramid build in the representation the mode reads) plus
`iterations` lookups — and the table reports the time of that job and the bytes
the mode holds on the device (inputs + library + output).  Inputs are synthetic:
random feature vectors as in the paper, feature maps of width W and height
7 W / 16 (the shapes of the paper's table: 512 x 224 and so on), query
centroids = pixel grid + a smooth motion field of amplitude W / 10 + N(0, 0.5)
jitter redrawn for every lookup.  The paper's centroids come from RAFT on
Sintel; these stand in for them.

The last column cross-checks what was timed: the largest difference between the block mode's
output and the on-demand mode's (a plain fp32 evaluation of Eq. 1, one wave per query) for the last
lookup, as a fraction of the parity bound 1e-4 * max|C|.  Parity with the CPU oracle at these shapes
is a test of its own (tests/test_gpu_sweep_points.py).

The full-volume column is this library's reference mode: an untuned fp32 vector-ALU GEMM (about 46
TFLOP/s) and an unfused pooling pass.  A tuned dense volume would be several times faster, so the
width at which block mode overtakes it in this table flatters block mode; the memory columns do not
depend on that.

Usage (GPU machine, repository root):  python -m paper_2505_16942_amd.sweep [--quick]
Prints a markdown table.  With --backward it prints a second kind of table instead: one call of the lookup's
gradient (corr_sample_backward) over the same widths and feature dimensionalities, in both of its forms, beside one
lookup.
"""
from __future__ import annotations

import argparse
import sys
import time


def _case(width: int, D: int, seed: int):
    import numpy as np
    import torch
    from . import synth
    H = max(width * 7 // 16, 8)
    W = width
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    f1 = torch.randn((1, D, H, W), device=dev, generator=g)
    f2 = torch.randn((1, D, H, W), device=dev, generator=g)
    rng = np.random.Generator(np.random.PCG64([seed, 3]))
    field = synth.smooth_field(rng, H, W, W / 10.0)
    ys, xs = np.meshgrid(np.arange(H, dtype=np.float64), np.arange(W, dtype=np.float64), indexing="ij")
    cs = []
    for t in range(2):
        fl = field + rng.normal(0.0, 0.5, (2, H, W))
        c = np.stack([xs + fl[0], ys + fl[1]])[None].astype(np.float32)
        cs.append(torch.from_numpy(c).to(dev))
    return H, W, f1, f2, cs


def _run_point(width: int, iters: int, D: int, L: int = 4, r: int = 4, reps_timed: int = 2):
    """Returns {mode: (ms, bytes) or ("OOM", bytes)} for block (bf16x3), block_bf16, ondemand, fullvolume."""
    import torch
    from . import binding as cb
    H, W, f1, f2, cs = _case(width, D, 7000 + width + D)
    out = torch.empty((1, L * 81, H, W), dtype=torch.float32, device=f1.device)
    caller = (f1.numel() + f2.numel() + out.numel() + 2 * H * W) * 4
    res = {}
    last = {}
    modes = [("block", cb.CORR_MODE_BLOCK, cb.CORR_PREC_BF16X3, cb.CORR_REP_SPLIT),
             ("block_bf16", cb.CORR_MODE_BLOCK, cb.CORR_PREC_BF16, cb.CORR_REP_BF16),
             ("ondemand", cb.CORR_MODE_ONDEMAND, cb.CORR_PREC_BF16X3, cb.CORR_REP_F32),
             ("fullvolume", cb.CORR_MODE_FULLVOLUME, cb.CORR_PREC_BF16X3, cb.CORR_REP_F32)]
    for name, mode, prec, reps in modes:
        if mode == cb.CORR_MODE_FULLVOLUME:
            need = cb.corr_full_volume_bytes(1, H, W, L)
            free_b, _ = torch.cuda.mem_get_info()
            if need + (1 << 30) > free_b:
                res[name] = ("OOM", need + caller)
                continue
        pyr = cb.corr_pyramid_build(f1, f2, L=L, reps=reps)

        def job():
            cb.corr_pyramid_build(f1, f2, L=L, reps=reps, pyramid=pyr)
            for t in range(iters):
                cb.corr_sample(f1, pyr, cs[t & 1], r=r, out=out, mode=mode, prec=prec)

        try:
            job()                                   # warm-up (and the volume allocation of full-volume mode)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps_timed):
                job()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / reps_timed
            res[name] = (ms, pyr.bytes() + caller)
            if name in ("block", "ondemand"):
                last[name] = out.clone()
        except cb.CorrError as e:
            if e.status != cb.CORR_ERR_OOM:
                raise
            res[name] = ("OOM", cb.corr_full_volume_bytes(1, H, W, L) + caller)
        pyr.destroy()
        torch.cuda.empty_cache()
    if "block" in last and "ondemand" in last:
        maxc = float(last["ondemand"].abs().max())
        res["check"] = float((last["block"] - last["ondemand"]).abs().max()) / (1e-4 * max(maxc, 1e-30))
    return H, W, res


def _backward_point(width: int, D: int, calls: int = 5):
    """(H, W, ms of one lookup, ms of one gradient call in the work-item form, ms in the one-wave-per-query form)."""
    import torch
    from . import binding as cb
    H, W, f1, f2, cs = _case(width, D, 11)
    dev = f1.device
    d_out = torch.randn((1, 4 * 81, H, W), device=dev)
    pyr = cb.corr_pyramid_build(f1, f2, L=4, reps=cb.CORR_REP_F32 | cb.CORR_REP_SPLIT)
    ws = torch.empty(cb.corr_backward_workspace_bytes(1, H, W, D, 4) // 4, device=dev)
    g1, g2 = torch.empty_like(f1), torch.empty_like(f1)
    out = cb.corr_sample(f1, pyr, cs[0])

    def timed(fn, n):
        fn(); fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    res = [timed(lambda: cb.corr_sample(f1, pyr, cs[0], out=out), calls)]
    try:
        for form, n in ((cb.CORR_BACKWARD_ITEMS, calls), (cb.CORR_BACKWARD_QUERIES, 2)):
            cb.corr_debug_set_backward_form(form)
            res.append(timed(lambda: cb.corr_sample_backward(pyr, cs[0], d_out, d_fmap1=g1, d_fmap2=g2, workspace=ws), n))
    finally:
        cb.corr_debug_set_backward_form(cb.CORR_BACKWARD_ITEMS)
    pyr.destroy()
    return H, W, res[0], res[1], res[2]


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--quick", action="store_true", help="fewer and smaller points")
    ap.add_argument("--backward", action="store_true", help="the gradient's table instead of the lookup's")
    args = ap.parse_args(argv)
    import torch
    from . import binding as cb
    if not torch.cuda.is_available():
        print("sweep: no GPU visible", file=sys.stderr)
        return 1
    cb.load_library()
    if args.backward:
        pts = [("Input width", w, (w, 256)) for w in ((32, 128, 512) if args.quick else (32, 64, 128, 256, 512, 1024))]
        pts += [("Feature dimensionality", d, (512, d)) for d in ((64,) if args.quick else (64, 128, 512))]
        print("| variable | value | map HxW | one lookup (block bf16x3) ms | gradient, work items ms | gradient, one wave per query ms |")
        print("|---|---|---|---|---|---|")
        for var, val, (w, d) in pts:
            H, W, fwd, items, queries = _backward_point(w, d)
            print("| %s | %d | %dx%d | %.3f | %.3f | %.3f |" % (var, val, H, W, fwd, items, queries), flush=True)
        return 0
    base_w, base_it, base_d = 512, 32, 256
    if args.quick:
        points = [("Input width", w, (w, base_it, base_d)) for w in (32, 128, 512)]
        points += [("Iterations", 8, (base_w, 8, base_d)), ("Feature dimensionality", 64, (base_w, base_it, 64))]
    else:
        points = [("Input width", w, (w, base_it, base_d)) for w in (32, 64, 128, 256, 512, 1024, 2048)]
        points += [("Iterations", n, (base_w, n, base_d)) for n in (1, 8, 16, 24, 32)]
        points += [("Feature dimensionality", d, (base_w, base_it, d)) for d in (64, 128, 256, 512, 1024)]
    print("| variable | value | map HxW | block bf16x3 ms | block bf16 ms | on-demand ms | full volume ms | "
          "block MB | on-demand MB | full volume MB | block vs on-demand, max diff / bound |")
    print("|---|---|---|---|---|---|---|---|---|---|---|")
    for var, val, (w, it, d) in points:
        H, W, res = _run_point(w, it, d)

        def ms(k):
            v = res[k][0]
            return v if isinstance(v, str) else "%.2f" % v

        def mb(k):
            return "%.0f" % (res[k][1] / 1e6)

        print("| %s | %d | %dx%d | %s | %s | %s | %s | %s | %s | %s | %.3f |" % (
            var, val, H, W, ms("block"), ms("block_bf16"), ms("ondemand"), ms("fullvolume"),
            mb("block"), mb("ondemand"), mb("fullvolume"), res.get("check", float("nan"))), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())

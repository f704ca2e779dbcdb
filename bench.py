"""Benchmark of the FP8 hot path on one MI355X.

A "step" is one pass of the whole path over one synthetic batch of a benchmark config (default:
config 5, the 8B-scale block): for every linear layer the just-in-time casts of X, W, dY
(abs-max -> scale -> cast in one call) and the forward (NT) / data-gradient (NN) / weight-gradient (TN) FP8
GEMMs, then the casts of Q, K, V, dO and FP8 causal
attention forward and backward.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line: metric = FP8 TFLOP/s of the whole step (GEMM + attention FLOPs over the
step's wall time, casts included in the time), plus
  roofline      -- the dominant kernel (the FP8 GEMM), timed per launch with HIP events on the
                   launch stream inside the timed region,
  cpu_baseline  -- the CPU oracle timed on a bounded sample of the same workload,
  kernels       -- the same per-class figures for attention and the just-in-time cast, from a second set of
                   passes outside the timed region (event pairs around small kernels cost as much
                   as the kernels themselves and would distort the headline figure).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP8_TFLOPS = 5033.0     # 256 CU x 4 SIMD x 2048 FLOP/clk x 2.4 GHz (dense FP8 MFMA)
PEAK_HBM_GBS = 8000.0
# HBM bytes per fp8_gemm_kernel launch (average over the step's 15 launches), from two rocprofv3 --pmc
# runs of this script (FETCH_SIZE, WRITE_SIZE), each scaled by the reading of a plain 1 GiB copy:
# 668 MB read + 123 MB written.  Only measured for the default workload.
MEASURED_GEMM_TRAFFIC_BYTES = {5: 7.905e8}


def cpu_baseline(cfg):
    """The oracle, as it stands, on a bounded sample: output rows of the first linear's forward GEMM."""
    import numpy as np
    from oracle import fp8, gemm, scaling
    from paper_2505_20524_amd import synth
    lin = cfg.linears[0] if cfg.linears else None
    if lin is None:
        return None
    t = synth.linear_tensors(cfg, 0, want=("X", "W"))
    q = {}
    for name in ("X", "W"):
        rho, rinv = scaling.compute_scale(scaling.amax(t[name]), fp8.E4M3)
        q[name] = (scaling.quantize(t[name], rho, fp8.E4M3), rinv)
    rows = np.arange(0, lin.M, max(1, lin.M // 256))[:256]
    t0 = time.perf_counter()
    reps = 0
    while True:
        gemm.fp8_gemm_rows(gemm.NT, q["X"][0], fp8.E4M3, q["X"][1], q["W"][0], fp8.E4M3, q["W"][1], rows)
        reps += 1
        dt = time.perf_counter() - t0
        if dt > 10.0 or reps >= 50:
            break
    flops = 2.0 * len(rows) * lin.N * lin.K * reps
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d of %d output rows of the %s forward GEMM (N=%d, K=%d), decode + float64 matmul, %d repeats, %.1f s"
                      % (len(rows), lin.M, lin.name, lin.N, lin.K, reps, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--vendor-context", action="store_true",
                    help="also time the vendor library's FP8 GEMM (torch._scaled_mm) on the forward shapes: context only, "
                         "never on the path and never part of `value`")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (no collectives are on the path); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2505_20524_amd import block, fog, synth
    fog.load()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.config]
    blk = block.Block(cfg)
    torch.cuda.synchronize()

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        blk.step()
    torch.cuda.synchronize()
    # Timed region: exactly `steps` passes.  HIP events (recorded on the launch stream, torch's current
    # stream) bracket the launches of the dominant kernel, the FP8 GEMM, inside this region: one pair around
    # the three back-to-back products of each linear layer, whose time divided by three is the launch average.  The other
    # kernel classes are timed the same way in a second, untimed set of passes: an event pair costs
    # several microseconds, and 74 of them per step would lower the headline figure by several per cent.
    dominant = "gemm" if blk.linears else "attn_fwd"
    timer = block.EventTimer(only={dominant})
    t0 = time.perf_counter()
    for _ in range(args.steps):
        blk.step(timer)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    value = blk.flops / (ms_per_step * 1e-3) / 1e12
    others = block.EventTimer()
    for _ in range(args.steps):
        blk.step(others)
    torch.cuda.synchronize()
    summ = others.summary()
    summ[dominant] = timer.summary()[dominant]
    kernels = {}
    for kind, (n, work, ms) in summ.items():
        if kind in ("gemm", "attn_fwd", "attn_bwd"):
            ach = work / (ms * 1e-3) / 1e12
            kernels[kind] = {"launches_per_step": n // args.steps, "avg_launch_ms": ms / n, "achieved": ach,
                             "unit": "TFLOP/s", "frac": ach / PEAK_FP8_TFLOPS, "in_timed_region": kind == dominant}
        else:
            ach = work / (ms * 1e-3) / 1e9
            kernels[kind] = {"launches_per_step": n // args.steps, "avg_launch_ms": ms / n, "achieved": ach,
                             "unit": "GB/s", "frac": ach / PEAK_HBM_GBS, "in_timed_region": False}
    # The kurtosis monitor (a diagnostic, not a step of the training path): timed on its own, after the
    # timed region, over the activation inputs of every linear layer.
    if blk.linears:
        kout = torch.zeros(1, device="cuda")
        kt = block.EventTimer()
        for rep in range(4):
            for l in blk.linears:
                if rep:
                    kt.begin("kurtosis", l.X.x.numel() * 2)
                fog.kurtosis(l.X.x, kout)
                if rep:
                    kt.end()
        torch.cuda.synchronize()
        n, work, ms = kt.summary()["kurtosis"]
        kernels["kurtosis_monitor"] = {"launches": n, "avg_launch_ms": ms / n, "achieved": work / (ms * 1e-3) / 1e9,
                                       "unit": "GB/s", "frac": work / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "in_timed_step": False}
    # The cast fused with the transpose (the arrangement for a weight gradient computed as NT on transposed
    # copies).  The timed step does not need it: its weight gradients are TN products on the row-major casts,
    # the kernel gathering the contraction index with the transposing LDS read.  Timed on its own over the
    # activations and output gradients of every linear layer (2 B read + 2 B written per element).
    if blk.linears and not blk.linears[0].transposed_wgrad:
        tt = block.EventTimer()
        for l in blk.linears:
            for c in (l.X, l.dY):
                rows, cols = c.x.shape
                qT = torch.empty((cols, rows), dtype=torch.uint8, device="cuda")
                for rep in range(3):
                    if rep:
                        tt.begin("cast_transpose", 4 * rows * cols)
                    fog.quantize(c.x, c.fmt, c.scale, q=c.q, qT=qT)
                    if rep:
                        tt.end()
                del qT
        torch.cuda.synchronize()
        n, work, ms = tt.summary()["cast_transpose"]
        kernels["cast_transpose"] = {"launches": n, "avg_launch_ms": ms / n, "achieved": work / (ms * 1e-3) / 1e9,
                                     "unit": "GB/s", "frac": work / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "in_timed_step": False}
    # The fused QK-RMSNorm + cast producer (an alternative source of the Q / K bytes, not part of the timed
    # step, whose casts are the plain per-tensor ones): timed on its own over the step's Q and K tensors.
    if blk.attn is not None:
        nt = block.EventTimer()
        one = torch.full((1,), 39.0, device="cuda")
        am = torch.zeros(1, device="cuda")
        for rep in range(4):
            for name in ("Q", "K"):
                c = blk.attn.c[name]
                if rep:
                    nt.begin("qknorm", 3 * c.x.numel())
                fog.rmsnorm_quantize(c.x, fog.E4M3, one, c.q, gain=1.0, amax_out=am)
                if rep:
                    nt.end()
        torch.cuda.synchronize()
        n, work, ms = nt.summary()["qknorm"]
        kernels["qknorm_cast"] = {"launches": n, "avg_launch_ms": ms / n, "achieved": work / (ms * 1e-3) / 1e9,
                                  "unit": "GB/s", "frac": work / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "in_timed_step": False}
    # The fused xIELU + cast producer (the input of the second feed-forward GEMM in the FOG-max variant; not part
    # of the timed step): timed on its own over the activation input of the last linear layer (the down projection).
    if blk.linears:
        c = blk.linears[-1].X
        xt = block.EventTimer()
        am = torch.zeros(1, device="cuda")
        for rep in range(4):
            if rep:
                xt.begin("xielu", 3 * c.x.numel())
            fog.xielu_quantize(c.x, 0.8, 0.8, fog.E4M3, c.scale, c.q, amax_out=am)
            if rep:
                xt.end()
        torch.cuda.synchronize()
        n, work, ms = xt.summary()["xielu"]
        kernels["xielu_cast"] = {"launches": n, "avg_launch_ms": ms / n, "achieved": work / (ms * 1e-3) / 1e9,
                                 "unit": "GB/s", "frac": work / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "in_timed_step": False}
    context = None
    if args.vendor_context and blk.linears:
        # Context only: the same forward products (NT, E4M3 x E4M3 -> bf16) through the vendor library, next to
        # this library's kernel on identical operands, each timed over 10 back-to-back launches.
        def timed(fn, iters=10):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(iters):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / iters
        one = torch.ones(1, device="cuda")
        context = {"kind": "vendor FP8 GEMM via torch._scaled_mm, forward shapes, TFLOP/s", "shapes": []}
        for l in blk.linears:
            M, N, K = l.lin.M, l.lin.N, l.lin.K
            a8, b8 = l.X.q.view(torch.float8_e4m3fn), l.W.q.view(torch.float8_e4m3fn)
            entry = {"M": M, "N": N, "K": K}
            ms = timed(lambda: fog.fp8_gemm(fog.NT, M, N, K, l.X.q, fog.E4M3, one, l.W.q, fog.E4M3, one, l.Y))
            entry["this_library"] = 2.0 * M * N * K / ms / 1e9
            try:
                ms = timed(lambda: torch._scaled_mm(a8, b8.t(), scale_a=one, scale_b=one, out_dtype=torch.bfloat16))
                entry["vendor"] = 2.0 * M * N * K / ms / 1e9
            except Exception as e:      # the vendor path is optional context
                entry["vendor"] = None
                entry["vendor_error"] = repr(e)[:200]
            context["shapes"].append(entry)
    g = kernels.get("gemm") or kernels.get("attn_fwd")
    roofline = {"bound": "mfma", "kernel": "fp8_gemm_kernel" if "gemm" in kernels else "attn_fwd_kernel",
                "achieved": g["achieved"], "peak": PEAK_FP8_TFLOPS, "unit": "TFLOP/s", "frac": g["frac"],
                "traffic": MEASURED_GEMM_TRAFFIC_BYTES.get(cfg.cid) if "gemm" in kernels else None, "launches_per_step": g["launches_per_step"], "avg_launch_ms": g["avg_launch_ms"]}

    out = {
        "metric": "FP8 TFLOP/s (block GEMMs fwd+dgrad+wgrad + FP8 causal attention fwd+bwd, casts in the timed step)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8_e4m3_e5m2", "data": "synthetic",
        "config": {"workload": "config %d: %s" % (cfg.cid, cfg.label), "gflop_per_step": blk.flops / 1e9},
        "frac_of_fp8_peak": value / PEAK_FP8_TFLOPS,
        "roofline": roofline, "kernels": kernels,
    }
    if context is not None:
        out["context"] = context
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

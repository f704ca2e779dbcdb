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
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP8_TFLOPS = 5033.0     # 256 CU x 4 SIMD x 2048 FLOP/clk x 2.4 GHz (dense FP8 MFMA)
PEAK_HBM_GBS = 8000.0


def _host_threads():
    """(threads the BLAS behind numpy uses, cores this process may run on)."""
    affinity = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    try:
        from threadpoolctl import threadpool_info
        blas = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        blas = affinity
    return min(blas, affinity), affinity


def cpu_baseline(cfg):
    """The oracle, as it stands, timed on bounded samples of the same workload, one per kernel class:
    output rows of the first linear layer's forward GEMM (the headline figure, in the metric's unit), the
    abs-max and the cast of a slice of that layer's activations, and one (batch, head) pair of attention
    forward and backward.  About 20-30 s of CPU work in all."""
    import numpy as np
    from oracle import attention, bf16, fp8, gemm, scaling
    from paper_2505_20524_amd import synth
    blas_threads, affinity = _host_threads()
    classes = {}
    out = None
    if cfg.linears:
        lin = cfg.linears[0]
        t = synth.linear_tensors(cfg, 0, want=("X", "W"))
        # casts: a slice of X (the oracle's cast is element-wise numpy, one thread)
        rows = max(1, min(lin.M, (1 << 22) // lin.K))
        xs = t["X"][:rows]
        t0 = time.perf_counter()
        reps = 0
        while True:
            a = scaling.amax(xs)
            reps += 1
            dt_a = time.perf_counter() - t0
            if dt_a > 1.0 or reps >= 50:
                break
        classes["amax"] = {"value": 2.0 * xs.size * reps / dt_a / 1e9, "unit": "GB/s", "cores": 1,
                           "sample": "%d of %d rows of %s X, %d repeats, %.2f s" % (rows, lin.M, lin.name, reps, dt_a)}
        rho, _ = scaling.compute_scale(a, fp8.E4M3)
        t0 = time.perf_counter()
        reps = 0
        while True:
            scaling.quantize(xs, rho, fp8.E4M3)
            reps += 1
            dt_q = time.perf_counter() - t0
            if dt_q > 3.0 or reps >= 20:
                break
        classes["cast"] = {"value": 3.0 * xs.size * reps / dt_q / 1e9, "unit": "GB/s", "cores": 1,
                           "sample": "%d of %d rows of %s X (2 B read + 1 B written per element), %d repeats, %.2f s"
                                     % (rows, lin.M, lin.name, reps, dt_q)}
        q = {}
        for name in ("X", "W"):
            rho, rinv = scaling.compute_scale(scaling.amax(t[name]), fp8.E4M3)
            # whole operands, cast on row chunks (bounds the oracle's temporaries)
            step = max(1, (1 << 22) // t[name].shape[1])
            q[name] = (np.concatenate([scaling.quantize(t[name][r:r + step], rho, fp8.E4M3) for r in range(0, t[name].shape[0], step)]), rinv)
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
        classes["gemm"] = {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": blas_threads,
                           "sample": "%d of %d output rows of the %s forward GEMM (N=%d, K=%d), decode + float64 matmul, %d repeats, %.1f s"
                                     % (len(rows), lin.M, lin.name, lin.N, lin.K, reps, dt)}
        out = dict(classes["gemm"])
    if cfg.attn is not None:
        a = cfg.attn
        rng = np.random.default_rng(0)
        S = min(a.S, 4096)
        # one head of synthetic codes of the config's sequence length (the oracle's cost does not depend on the values)
        codes = lambda: rng.integers(0, 0x78, size=(S, a.D)).astype(np.uint8) | (rng.integers(0, 2, size=(S, a.D)).astype(np.uint8) << 7)
        Q8, K8, V8, dO8 = codes(), codes(), codes(), codes()
        sq = np.float32(1.0 / 64)
        s = 1.0 / math.sqrt(a.D)
        t0 = time.perf_counter()
        O, lse, _ = attention.attn_fwd_head(Q8, K8, V8, sq, sq, sq, s, 448.0, True)
        dt_f = time.perf_counter() - t0
        fl = 4.0 * S * S * a.D / 2
        classes["attn_fwd"] = {"value": fl / dt_f / 1e12, "unit": "TFLOP/s", "cores": blas_threads,
                               "sample": "one (batch, head) pair, S=%d, D=%d, causal, %.2f s (FLOPs counted on the causal half)" % (S, a.D, dt_f)}
        O_bits = bf16.f64_to_bits_rne(O)
        dO_bits = bf16.f64_to_bits_rne(fp8.decode(dO8, fp8.E5M2) * 1e-4)
        t0 = time.perf_counter()
        attention.attn_bwd_head(Q8, K8, V8, sq, sq, sq, O_bits, dO_bits, dO8, np.float32(1e-4), lse.astype(np.float32), s, 448.0, 1024.0, True)
        dt_b = time.perf_counter() - t0
        classes["attn_bwd"] = {"value": 2.5 * fl / dt_b / 1e12, "unit": "TFLOP/s", "cores": blas_threads,
                               "sample": "the same pair, backward, %.2f s" % dt_b}
        if out is None:
            out = dict(classes["attn_fwd"])
    if out is None:
        return None
    out["kind"] = "oracle"
    out["affinity_cores"] = affinity
    out["classes"] = classes
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--cast-batching", choices=["layer", "weights", "step"], default="layer",
                    help="how the just-in-time casts are grouped into batched calls (see block.Block)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--vendor-context", action="store_true",
                    help="also time the vendor library's FP8 GEMM (torch._scaled_mm) on the forward shapes: context only, "
                         "never on the path and never part of `value`")
    ap.add_argument("--ceilings", action="store_true",
                    help="also measure what the GPU sustains: a register-resident FP8 matrix-instruction loop on several operand "
                         "bit patterns (constant, small codes, random bytes, the step's own operands) and plain HBM read / copy rates")
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
    blk = block.Block(cfg, cast_batching=args.cast_batching)
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
    summ = others.summary(drop_outliers=True)
    # The same step under delayed scaling (the recipe of the paper's runs): every cast is one pass with the scale
    # from its abs-max history.  A second figure, not the headline (the metric is quoted on just-in-time scaling).
    for _ in range(max(args.warmup, 2)):
        blk.step(delayed=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        blk.step(delayed=True)
    torch.cuda.synchronize()
    delayed_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    dl = block.EventTimer(only={"cast_delayed"})
    for _ in range(args.steps):
        blk.step(dl, delayed=True)
    torch.cuda.synchronize()
    summ["cast_delayed"] = dl.summary(drop_outliers=True)["cast_delayed"]
    summ[dominant] = timer.summary()[dominant]
    kernels = {}
    for kind, (n, work, ms) in summ.items():
        if kind in ("gemm", "attn_fwd", "attn_bwd"):
            ach = work / (ms * 1e-3) / 1e12
            kernels[kind] = {"launches_per_step": max(1, round(n / args.steps)), "avg_launch_ms": ms / n, "achieved": ach,
                             "unit": "TFLOP/s", "frac": ach / PEAK_FP8_TFLOPS, "in_timed_region": kind == dominant}
        else:
            ach = work / (ms * 1e-3) / 1e9
            kernels[kind] = {"launches_per_step": max(1, round(n / args.steps)), "avg_launch_ms": ms / n, "achieved": ach,
                             "unit": "GB/s", "frac": ach / PEAK_HBM_GBS, "in_timed_region": False}
    # Figures of kernels that are not steps of the timed path, each timed on its own after the timed region
    # (first repetition untimed): jobs = [(algorithmic bytes, call), ...].
    def side_figure(key, jobs, reps=4):
        # one event pair around a whole pass over the jobs, launched back to back: an event between two launches
        # costs a gap of 6-10 us on the stream, a fifth of what these kernels take on the step's tensors
        t = block.EventTimer()
        total = sum(work for work, _ in jobs)
        for rep in range(reps):
            if rep:
                t.begin(key, total, launches=len(jobs))
            for _, fn in jobs:
                fn()
            if rep:
                t.end()
        torch.cuda.synchronize()
        n, work, ms = t.summary()[key]
        kernels[key] = {"launches": n, "avg_launch_ms": ms / n, "achieved": work / (ms * 1e-3) / 1e9,
                        "unit": "GB/s", "frac": work / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "in_timed_step": False}

    # The step's just-in-time casts again, back to back without the products between them.  Inside the step the abs-max
    # pass that follows a GEMM also pays for the write-back of that GEMM's output (up to 235 MB of dirty lines leave
    # the caches while it streams); alone, the same launches show what the cast kernels themselves sustain.
    alone = block.EventTimer(only={"cast_jit"})
    for rep in range(4):
        per_layer = [] if blk.cast_batching == "step" else [l.casts for l in blk.linears] + ([blk.attn.casts] if blk.attn else [])
        for b in blk.pre + per_layer:
            b.run(alone if rep else None)
    torch.cuda.synchronize()
    n, work, ms = alone.summary()["cast_jit"]
    kernels["cast_jit_without_gemms"] = {"launches": n, "avg_launch_ms": ms / n, "achieved": work / (ms * 1e-3) / 1e9, "unit": "GB/s",
                                         "frac": work / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "in_timed_step": False}
    am = torch.zeros(1, device="cuda")
    if blk.linears:
        # The kurtosis monitor (a diagnostic) over the activation inputs of every linear layer, alone and with
        # the abs-max of delayed scaling taken from the same read (2 B per element either way).
        kout = torch.zeros(1, device="cuda")
        side_figure("kurtosis_monitor", [(l.X.x.numel() * 2, lambda l=l: fog.kurtosis(l.X.x, kout)) for l in blk.linears])
        side_figure("kurtosis_with_amax", [(l.X.x.numel() * 2, lambda l=l: fog.kurtosis(l.X.x, kout, amax_out=am)) for l in blk.linears])
    # The cast fused with the transpose (the arrangement for a weight gradient computed as NT on transposed
    # copies).  The timed step does not need it: its weight gradients are TN products on the row-major casts,
    # the kernel gathering the contraction index with the transposing LDS read.  Over the activations and
    # output gradients of every linear layer (2 B read + 2 B written per element).
    if blk.linears and not blk.linears[0].transposed_wgrad:
        big = max(c.x.numel() for l in blk.linears for c in (l.X, l.dY) if c is not None)
        qT_store = torch.empty(big, dtype=torch.uint8, device="cuda")
        jobs = []
        for l in blk.linears:
            for c in (l.X, l.dY):
                if c is None:
                    continue
                rows, cols = c.x.shape
                qT = qT_store[: rows * cols].view(cols, rows)
                jobs.append((4 * rows * cols, lambda c=c, qT=qT: fog.quantize(c.x, c.fmt, c.scale, q=c.q, qT=qT)))
        side_figure("cast_transpose", jobs, reps=3)
        del qT_store, jobs
    # Fused producers of the casts (alternative sources of the FP8 bytes, not part of the timed step, whose casts
    # are the plain per-tensor ones).  QK-RMSNorm and tanh_alpha over the step's Q and K tensors; xIELU and GeLU
    # over the activation input of the last linear layer (the down projection); 2 B read + 1 B written per element.
    if blk.attn is not None:
        rho_qk = torch.full((1,), 39.0, device="cuda")
        rho_max = torch.full((1,), 448.0, device="cuda")
        qk = [blk.attn.c[name] for name in ("Q", "K")]
        side_figure("qknorm_cast", [(3 * c.x.numel(), lambda c=c: fog.rmsnorm_quantize(c.x, fog.E4M3, rho_qk, c.q, gain=1.0, amax_out=am))
                                    for c in qk])
        side_figure("tanh_cast", [(3 * c.x.numel(), lambda c=c: fog.tanh_quantize(c.x, 0.5, fog.E4M3, rho_max, c.q, amax_out=am))
                                  for c in qk])
    if blk.linears:
        c = blk.linears[-1].X
        side_figure("xielu_cast", [(3 * c.x.numel(), lambda: fog.xielu_quantize(c.x, 0.8, 0.8, fog.E4M3, c.scale, c.q, amax_out=am))])
        side_figure("gelu_cast", [(3 * c.x.numel(), lambda: fog.gelu_quantize(c.x, fog.E4M3, c.scale, c.q, amax_out=am))])
        # Post-RMSNorm + residual + cast over the output of the last linear layer (the sub-layer output y) and the
        # first layer's activation input as the residual stream x, updated into a buffer of its own:
        # 2 + 2 B read, 2 + 1 B written per element.
        y, xres = blk.linears[-1].Y, blk.linears[0].X
        if y.shape == xres.x.shape:
            gamma = torch.full((y.shape[1],), 1.0 / math.sqrt(32.0), device="cuda")
            xnew = torch.empty_like(y)
            side_figure("postnorm_residual_cast", [(7 * y.numel(), lambda: fog.postnorm_residual_quantize(
                xres.x, y, gamma, fog.E4M3, xres.scale, xnew, q=xres.q, amax_out=am))])
            del xnew
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
            if M % 256 == 0 and N % 256 == 0:
                # the same launch with every tile's epilogue left out (measurement helper): what hiding the epilogues could gain
                ms = timed(lambda: fog.probe_gemm_products_only(M, N, K, l.X.q, one, l.W.q, one, l.Y))
                entry["this_library_products_only"] = 2.0 * M * N * K / ms / 1e9
            try:
                ms = timed(lambda: torch._scaled_mm(a8, b8.t(), scale_a=one, scale_b=one, out_dtype=torch.bfloat16))
                entry["vendor"] = 2.0 * M * N * K / ms / 1e9
            except Exception as e:      # the vendor path is optional context
                entry["vendor"] = None
                entry["vendor_error"] = repr(e)[:200]
            context["shapes"].append(entry)
    ceilings = None
    if args.ceilings:
        # What the part sustains, next to the published peaks the fractions above are taken against.  The matrix
        # instruction issues every 64 cycles whatever its operands are; the clock it runs at depends on the power the
        # operand bits draw, so the same loop is timed on four 64 KB operand patterns.
        gen = torch.Generator(device="cuda"); gen.manual_seed(5)
        rnd = lambda lo, hi: torch.randint(lo, hi, (65536,), dtype=torch.uint8, device="cuda", generator=gen)
        sign = lambda: torch.randint(0, 2, (65536,), dtype=torch.uint8, device="cuda", generator=gen) << 7
        patterns = {"one constant code (1.0)": torch.full((65536,), 0x38, dtype=torch.uint8, device="cuda"),
                    "codes of small magnitude, random sign (0x20-0x4f)": rnd(0x20, 0x50) | sign(),
                    "uniformly random finite codes": rnd(0, 0x7F) | sign()}
        if blk.linears:
            l0 = blk.linears[0]
            patterns["the step's own operands (first 32 KB of X~ and of W~ of %s)" % l0.lin.name] = torch.cat(
                [l0.X.q.reshape(-1)[:32768], l0.W.q.reshape(-1)[:32768]]).contiguous()
        sink = torch.empty(1024 * 512 + 4096, device="cuda")
        ceilings = {"mfma_loop": {}}
        for name, pat in patterns.items():
            fog.probe_mfma_rate(pat, 2000, sink)
            tf, ghz = fog.probe_mfma_rate(pat, 20000, sink)
            ceilings["mfma_loop"][name] = {"tflops": tf, "frac_of_peak": tf / PEAK_FP8_TFLOPS, "mfma_clock_ghz": ghz}
        # The attention forward's instruction mix without any memory traffic (see include/fog_probe.h): how far the matrix
        # cores and the vector ALU overlap on this part, at one to three waves per SIMD.
        ceilings["attention_loop_ns_per_wave_block"] = {}
        for wps in (1, 2, 3):
            t_all, t_mfma, t_valu, t_ilv = (fog.probe_attention_loop(w, wps, 3000, sink) for w in (0, 1, 2, 3))
            ceilings["attention_loop_ns_per_wave_block"]["%d waves per SIMD" % wps] = {
                "everything": t_all, "matrix instructions only": t_mfma, "softmax arithmetic only": t_valu,
                "everything, P V products dealt out between the softmax groups": t_ilv,
                "matrix_core_share_of_everything": t_mfma / t_all}
        # What one matrix instruction takes from the vector ALU of its own wave: shader cycles per slot (one matrix instruction
        # followed by n vector operations, order pinned), and the same vector operations alone.
        ceilings["cycles_per_mfma_slot"] = {}
        for op, name in ((0, "v_fma_f32"), (1, "v_exp_f32"), (2, "v_cvt_pk_fp8_f32"), (3, "softmax quarter group (fma, exp, add, max3 | convert)")):
            ceilings["cycles_per_mfma_slot"][name] = {
                "vector_ops": [0, 4, 8, 16, 32],
                "with_matrix_instruction": [fog.probe_mfma_coissue(op, n, True, 2000, sink) for n in (0, 4, 8, 16, 32)],
                "vector_ops_alone": [fog.probe_mfma_coissue(op, n, False, 2000, sink) for n in (0, 4, 8, 16, 32)]}
        # Whether one wave's vector work runs under ANOTHER wave's matrix instructions on the same SIMD: two waves per SIMD with
        # separate roles, each measured alone and while the other role (given more trips, so that it outlasts) is running.
        ceilings["cross_wave_cycles"] = {}
        for op, name in ((0, "v_fma_f32"), (1, "v_exp_f32"), (2, "v_cvt_pk_fp8_f32"), (3, "softmax quarter group (fma, exp, add, max3 | convert)")):
            n_ops, trips = 8, 2000
            _, v_alone = fog.probe_mfma_cross_wave(op, n_ops, 0, trips, sink)
            m_alone, _ = fog.probe_mfma_cross_wave(op, n_ops, trips, 0, sink)
            _, v_under = fog.probe_mfma_cross_wave(op, n_ops, int(trips * v_alone * 8 / 512 * 1.5) + trips, trips, sink)
            m_under, _ = fog.probe_mfma_cross_wave(op, n_ops, trips, int(trips * 512 / (v_alone * 8) * 1.5) + 64, sink)
            ceilings["cross_wave_cycles"][name] = {
                "vector_ops_per_group": n_ops, "vector_group_alone": v_alone, "vector_group_under_matrix_wave": v_under,
                "matrix_instruction_alone": m_alone, "matrix_instruction_under_vector_wave": m_under}
        # HBM: the abs-max kernel as a plain read (2 B per element) and a device copy, over buffers that do not fit the caches
        big = torch.empty(1 << 30, dtype=torch.int16, device="cuda")            # 2 GiB
        big.zero_()
        amx = torch.zeros(1, device="cuda")
        def rate(fn, nbytes, iters=5):
            fn(); torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(iters):
                fn()
            e1.record(); torch.cuda.synchronize()
            return nbytes * iters / (e0.elapsed_time(e1) * 1e-3) / 1e9
        ceilings["hbm_read_gbs"] = rate(lambda: fog.amax(big, amx), big.numel() * 2)
        half = big.numel() // 2
        ceilings["hbm_copy_gbs"] = rate(lambda: big[half:].copy_(big[:half]), half * 2 * 2)
        del big
    g = kernels.get("gemm") or kernels.get("attn_fwd")
    # HBM-side bytes per launch of the dominant kernel: read back from the rocprofv3 summary of this same command under
    # profiles/ (two --pmc runs, FETCH_SIZE and WRITE_SIZE, scaled by a plain copy; written by paper_2505_20524_amd.profile_summary);
    # null when the workload has no such summary.
    from paper_2505_20524_amd import profile_summary
    traffic = profile_summary.read_gemm_traffic(os.path.join(ROOT, "profiles"), cfg.cid) if "gemm" in kernels else None
    gemm_alg = None
    if blk.linears:
        # each operand read once (1 B per element), the bf16 result written once; forward-only layers launch one product
        total, launches = 0, 0
        for l in blk.linears:
            M, N, K = l.lin.M, l.lin.N, l.lin.K
            total += M * K + N * K + 2 * M * N
            launches += 1
            if l.backward:
                total += (M * N + N * K + 2 * M * K) + (M * N + M * K + 2 * N * K)
                launches += 2
        gemm_alg = total / float(launches)
    roofline = {"bound": "mfma", "kernel": "fp8_gemm_kernel" if "gemm" in kernels else "attn_fwd_kernel",
                "achieved": g["achieved"], "peak": PEAK_FP8_TFLOPS, "unit": "TFLOP/s", "frac": g["frac"],
                "traffic": traffic, "launches_per_step": g["launches_per_step"], "avg_launch_ms": g["avg_launch_ms"]}

    out = {
        "metric": "FP8 TFLOP/s (block GEMMs fwd+dgrad+wgrad + FP8 causal attention fwd+bwd, casts in the timed step)" if cfg.backward
                  else "FP8 TFLOP/s (forward GEMM, casts in the timed step)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8_e4m3_e5m2", "data": "synthetic",
        "config": {"workload": "config %d: %s" % (cfg.cid, cfg.label), "gflop_per_step": blk.flops / 1e9,
                   "cast_batching": args.cast_batching},
        "frac_of_fp8_peak": value / PEAK_FP8_TFLOPS, "gemm_algorithmic_bytes_per_launch": gemm_alg,
        "roofline": roofline, "kernels": kernels,
        "delayed_scaling": {"ms_per_step": delayed_ms, "value": blk.flops / (delayed_ms * 1e-3) / 1e12, "unit": "TFLOP/s",
                            "note": "same step with one-pass casts scaled from a 1024-entry abs-max history"},
    }
    if context is not None:
        out["context"] = context
    if ceilings is not None:
        out["ceilings"] = ceilings
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

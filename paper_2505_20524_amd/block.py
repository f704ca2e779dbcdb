"""Host-side driver of one pass of the hot path over a transformer block's GEMMs and attention.

For every linear layer Y = X W^T of the block: just-in-time per-tensor scaling (abs-max -> scale ->
cast) of X, W (E4M3) and dY (E5M2), the three tensors in one batched call (two launches), then the
three FP8 GEMMs (forward, data gradient, weight gradient; the weight gradient reads the row-major
casts, or transposed copies from the fused cast + transpose where a config asks for them).
For attention: casts of Q, K, V (E4M3) and dO (E5M2) in one batched call, FP8 attention forward and backward.
All arithmetic happens in the library's HIP kernels; this module only owns device buffers
(torch tensors) and the order of calls.  The elementwise operators between the GEMMs
(normalisation, activation, rotary embedding, residuals) are not part of the path: each GEMM
gets its own input tensors.
"""
import math

import numpy as np
import torch

from . import fog, synth

E4M3, E5M2 = fog.E4M3, fog.E5M2


def _dev_bits(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()


class Cast:
    """A bf16 tensor with its FP8 cast(s) and scalars, all resident in device memory."""

    def __init__(self, bits_dev, fmt, transpose):
        self.x = bits_dev
        self.fmt = fmt
        rows, cols = bits_dev.shape
        self.q = torch.empty((rows, cols), dtype=torch.uint8, device="cuda")
        self.qT = torch.empty((cols, rows), dtype=torch.uint8, device="cuda") if transpose else None
        self.amax = torch.zeros(1, device="cuda")
        self.scale = torch.ones(1, device="cuda")
        self.sinv = torch.ones(1, device="cuda")
        self.ws = torch.empty(fog.quantize_jit_workspace(), dtype=torch.uint8, device="cuda")
        self.history = None     # abs-max history of delayed scaling, allocated on first use
        self.bytes_jit = (5 + (1 if transpose else 0)) * rows * cols   # abs-max pass 2 B, cast pass 2 B in + 1 (+1 transposed) out

    def run(self, timer=None):
        """Just-in-time scaling in one call: abs-max pass (per-workgroup maxima), reduce + scale, cast."""
        if timer:
            timer.begin("cast_jit", self.bytes_jit)
        fog.quantize_jit(self.x, self.fmt, self.amax, self.scale, self.sinv, self.ws, q=self.q, qT=self.qT)
        if timer:
            timer.end()

    def run_delayed(self, timer=None):
        """Delayed scaling (Appendix E) in one launch: the abs-max the previous pass left behind enters the history
        (length 1024), the scale comes from the history's maximum, and ONE pass over the tensor casts with it and
        leaves this pass's abs-max for the next: 2 B read + 1 B written per element instead of 5.  Before the
        first abs-max exists the scale is 1."""
        if self.history is None:
            self.history = torch.zeros(1024, device="cuda")
            self.state = torch.zeros(fog.quantize_delayed_state(), dtype=torch.uint8, device="cuda")
            self.step = 0
        if timer:
            timer.begin("cast_delayed", self.bytes_jit - 2 * self.x.numel())
        fog.quantize_delayed(self.x, self.fmt, self.history, self.step, self.state, self.scale, self.sinv, q=self.q, qT=self.qT,
                             amax_prev=self.amax)
        if timer:
            timer.end()
        self.step += 1

    def run_delayed_two_calls(self):
        """The same flow through fog_scale_delayed and fog_quantize(..., amax_out): three launches, a shifting history."""
        if self.history is None:
            self.history = torch.zeros(1024, device="cuda")
            self.amax.zero_()
        fog.scale_delayed(self.history, self.amax, self.fmt, self.scale, self.sinv)
        fog.quantize(self.x, self.fmt, self.scale, q=self.q, qT=self.qT, amax_out=self.amax)

    def run_separate(self):
        """The same flow through the three calls fog_amax, fog_scale, fog_quantize (four launches)."""
        fog.amax(self.x, self.amax)
        fog.scale(self.amax, self.fmt, self.scale, self.sinv)
        fog.quantize(self.x, self.fmt, self.scale, q=self.q, qT=self.qT)


class CastBatch:
    """Just-in-time casts of several tensors in two launches (fog_quantize_jit_batch); tensors the batched call does
    not cover (a transposed copy wanted, a size that is not a multiple of 16) are cast one by one after it."""

    def __init__(self, casts):
        self.batched = [c for c in casts if c.qT is None and c.x.numel() % 16 == 0 and c.x.numel() > 0][:fog.CAST_BATCH_MAX]
        self.single = [c for c in casts if not any(c is b for b in self.batched)]
        self.jobs = fog.make_cast_jobs([(c.x, c.fmt, c.q, c.amax, c.scale, c.sinv) for c in self.batched])
        self.ws = torch.empty(max(fog.quantize_jit_batch_workspace(len(self.batched)), 16), dtype=torch.uint8, device="cuda")
        self.bytes = sum(c.bytes_jit for c in self.batched)
        self.delayed_jobs = None   # built on the first delayed-scaling pass

    def run(self, timer=None, delayed=False):
        if delayed:
            # one launch for the batch (fog_quantize_delayed_batch); what the batched call does not cover goes one by one
            if self.batched:
                if self.delayed_jobs is None:
                    for c in self.batched:
                        c.history = torch.zeros(1024, device="cuda")
                        c.state = torch.zeros(fog.quantize_delayed_state(), dtype=torch.uint8, device="cuda")
                    self.delayed_jobs = fog.make_delayed_jobs([(c.x, c.fmt, c.q, c.history, c.state, c.amax, c.scale, c.sinv) for c in self.batched])
                    self.delayed_step = 0
                if timer:
                    timer.begin("cast_delayed", sum(c.bytes_jit - 2 * c.x.numel() for c in self.batched), launches=len(self.batched))
                fog.quantize_delayed_batch(self.delayed_jobs, self.delayed_step)
                if timer:
                    timer.end()
                self.delayed_step += 1
            for c in self.single:
                c.run_delayed(timer)
            return
        if self.batched:
            if timer:
                timer.begin("cast_jit", self.bytes, launches=len(self.batched))
            fog.quantize_jit_batch(self.jobs, self.ws)
            if timer:
                timer.end()
        for c in self.single:
            c.run(timer)


class LinearStep:
    """Casts and the three GEMMs of one linear layer.

    transposed_wgrad=False (default): the weight gradient dW = dY~^T X~ is computed in the TN layout straight
    from the row-major casts; the kernel gathers the contraction index with the byte-transposing LDS read, so
    no transposed copy of X~ or dY~ is ever written.  transposed_wgrad=True: the casts also emit transposed
    copies (fused cast + transpose) and dW is an NT product on them, the arrangement for hardware without a
    transposing read; same results bit for bit."""

    def __init__(self, lin, tensors, transposed_wgrad=False, backward=True):
        self.lin = lin
        self.transposed_wgrad = transposed_wgrad
        self.backward = backward          # False: the forward product only (config 1), X and W are the only casts
        M, N, K = lin.M, lin.N, lin.K
        self.X = Cast(_dev_bits(tensors["X"]), E4M3, transpose=transposed_wgrad)
        self.W = Cast(_dev_bits(tensors["W"]), E4M3, transpose=False)
        self.Y = torch.empty((M, N), dtype=torch.int16, device="cuda")
        if not backward:
            self.dY = self.dX = self.dW = None
            self.flops = 2 * M * N * K
            self.casts = CastBatch([self.X, self.W])
            need = fog.fp8_gemm_workspace(fog.NT, M, N, K)
            self.gemm_ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
            return
        self.dY = Cast(_dev_bits(tensors["dY"]), E5M2, transpose=transposed_wgrad)
        self.dX = torch.empty((M, K), dtype=torch.int16, device="cuda")
        self.dW = torch.empty((N, K), dtype=torch.int16, device="cuda")
        self.flops = 3 * 2 * M * N * K
        self.casts = CastBatch([self.X, self.W, self.dY])
        # launches with fewer tiles than compute units are cut along the contraction through this workspace
        # (one buffer serves the layer's three products, which run one after the other)
        need = max(fog.fp8_gemm_workspace(fog.NT, M, N, K), fog.fp8_gemm_workspace(fog.NN, M, K, N),
                   fog.fp8_gemm_workspace(fog.NT if transposed_wgrad else fog.TN, N, K, M))
        self.gemm_ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None

    def run(self, timer=None, delayed=False):
        self.casts.run(timer, delayed)
        self.compute(timer)

    def compute(self, timer=None):
        lin = self.lin
        M, N, K = lin.M, lin.N, lin.K
        # The three products are launched back to back and bracketed by ONE event pair (an event between two
        # launches costs a gap of several microseconds on the stream): the pair's time is that of three launches.
        n_gemm = 3 if self.backward else 1
        if timer:
            timer.begin("gemm", n_gemm * 2 * M * N * K, launches=n_gemm)
        # forward  Y = X~ W~^T
        ws = self.gemm_ws
        fog.fp8_gemm(fog.NT, M, N, K, self.X.q, E4M3, self.X.sinv, self.W.q, E4M3, self.W.sinv, self.Y, workspace=ws)
        if not self.backward:
            if timer:
                timer.end()
            return
        # data gradient  dX = dY~ W~  (W~ is [N, K]: the contraction index N is its row index)
        fog.fp8_gemm(fog.NN, M, K, N, self.dY.q, E5M2, self.dY.sinv, self.W.q, E4M3, self.W.sinv, self.dX, workspace=ws)
        # weight gradient  dW = dY~^T X~  (contraction over the M tokens, the row index of both operands)
        if self.transposed_wgrad:
            fog.fp8_gemm(fog.NT, N, K, M, self.dY.qT, E5M2, self.dY.sinv, self.X.qT, E4M3, self.X.sinv, self.dW, workspace=ws)
        else:
            fog.fp8_gemm(fog.TN, N, K, M, self.dY.q, E5M2, self.dY.sinv, self.X.q, E4M3, self.X.sinv, self.dW, workspace=ws)
        if timer:
            timer.end()


class AttentionStep:
    def __init__(self, attn, tensors, softmax_scale=None):
        a = self.attn = attn
        n = a.B * a.H * a.S
        self.s = softmax_scale if softmax_scale is not None else 1.0 / math.sqrt(a.D)
        self.c = {name: Cast(_dev_bits(tensors[name].reshape(n, a.D)), E5M2 if name == "dO" else E4M3, False)
                  for name in ("Q", "K", "V", "dO")}
        self.casts = CastBatch([self.c[name] for name in ("Q", "K", "V", "dO")])
        self.O = torch.empty((n, a.D), dtype=torch.int16, device="cuda")
        self.lse = torch.empty(n, device="cuda")
        self.dQ, self.dK, self.dV = (torch.empty((n, a.D), dtype=torch.int16, device="cuda") for _ in range(3))
        self.scale_p = torch.full((1,), 448.0, device="cuda")
        self.amax_ds = torch.zeros(1, device="cuda")
        self.scale_ds = torch.ones(1, device="cuda")
        self.ws = torch.empty(max(fog.fp8_attn_workspace(a.B, a.H, a.S, a.D, True), 16), dtype=torch.uint8, device="cuda")
        self.flops_fwd = 4 * a.S * a.S * a.D // 2 * a.B * a.H      # causal: blocks at or below the diagonal
        self.flops_bwd = self.flops_fwd * 5 // 2
        self.flops = self.flops_fwd + self.flops_bwd

    def run(self, timer=None, delayed=False):
        self.casts.run(timer, delayed)
        self.compute(timer)

    def compute(self, timer=None):
        a, c = self.attn, self.c
        if timer:
            timer.begin("attn_fwd", self.flops_fwd)
        fog.fp8_attn_fwd(a.B, a.H, a.S, a.D, self.s, True, c["Q"].q, c["K"].q, c["V"].q, c["Q"].sinv, c["K"].sinv,
                         c["V"].sinv, self.scale_p, self.O, self.lse)
        if timer:
            timer.end()
        if timer:
            timer.begin("attn_bwd", self.flops_bwd)
        # delayed-style scale for dS: the abs-max this call reports sets the scale of the next call
        fog.fp8_attn_bwd(a.B, a.H, a.S, a.D, self.s, True, c["Q"].q, c["K"].q, c["V"].q, c["Q"].sinv, c["K"].sinv,
                         c["V"].sinv, self.O, c["dO"].x, c["dO"].q, c["dO"].sinv, self.lse, self.scale_p, self.scale_ds,
                         self.dQ, self.dK, self.dV, amax_ds=self.amax_ds, workspace=self.ws)
        if timer:
            timer.end()
        fog.scale(self.amax_ds, E5M2, self.scale_ds, None)


class Block:
    """All linears and the attention of one synthetic config, resident on the GPU.

    cast_batching says how the just-in-time casts are grouped into fog_quantize_jit_batch calls (two launches each):
      "layer"   -- one call per linear layer (X, W, dY) and one for attention (Q, K, V, dO), each right before its products;
      "weights" -- every weight of the block in one call at the start of the step (the weights all exist then), the
                   activations and gradients per layer as above;
      "step"    -- every tensor of the step in one call at its start.  The benchmark can do that because every product
                   has its own resident inputs; a training step can only for tensors that exist at that point."""

    def __init__(self, cfg, cast_batching="layer", attention_at=None):
        self.cfg = cfg
        self.cast_batching = cast_batching
        # position of attention among the linear layers (index of the layer it runs before; None = after the last)
        self.attention_at = attention_at
        # config 2 is stated with the fused cast + transpose for the weight gradient; the block configs leave the
        # arrangement open and use the TN product on the row-major casts
        self.linears = [LinearStep(lin, synth.linear_tensors(cfg, i, want=("X", "W", "dY") if cfg.backward else ("X", "W")),
                                   transposed_wgrad=(cfg.cid == 2), backward=cfg.backward)
                        for i, lin in enumerate(cfg.linears)]
        self.attn = AttentionStep(cfg.attn, synth.attention_tensors(cfg)) if cfg.attn is not None else None
        self.flops = sum(l.flops for l in self.linears) + (self.attn.flops if self.attn else 0)
        self.pre = []          # batches cast at the start of the step
        if cast_batching == "step":
            casts = [c for l in self.linears for c in (l.X, l.W, l.dY) if c is not None]
            if self.attn:
                casts += [self.attn.c[name] for name in ("Q", "K", "V", "dO")]
            self.pre = [CastBatch(casts[i:i + fog.CAST_BATCH_MAX]) for i in range(0, len(casts), fog.CAST_BATCH_MAX)]
        elif cast_batching == "weights":
            ws = [l.W for l in self.linears]
            self.pre = [CastBatch(ws[i:i + fog.CAST_BATCH_MAX]) for i in range(0, len(ws), fog.CAST_BATCH_MAX)]
            for l in self.linears:
                l.casts = CastBatch([c for c in (l.X, l.dY) if c is not None])
        elif cast_batching != "layer":
            raise ValueError(cast_batching)

    def step(self, timer=None, delayed=False):
        """One pass of the path; delayed=True scales every cast from its abs-max history instead of just in time."""
        for b in self.pre:
            b.run(timer, delayed)
        per_layer = self.cast_batching != "step"
        def attention():
            if per_layer:
                self.attn.casts.run(timer, delayed)
            self.attn.compute(timer)
        for i, l in enumerate(self.linears):
            if self.attn and self.attention_at == i:
                attention()
            if per_layer:
                l.casts.run(timer, delayed)
            l.compute(timer)
        if self.attn and (self.attention_at is None or self.attention_at >= len(self.linears)):
            attention()


class EventTimer:
    """Per-kernel-class HIP-event timing on the stream the library launches on (torch's current stream)."""

    def __init__(self, only=None):
        self.spans = []
        self._open = None
        self.only = only        # None: every kind; else the set of kinds to record (events cost time themselves)

    def begin(self, kind, work, launches=1):
        if self.only is not None and kind not in self.only:
            return
        e0 = torch.cuda.Event(enable_timing=True)
        e0.record()
        self._open = (kind, work, e0, launches)

    def end(self):
        if self._open is None:
            return
        kind, work, e0, launches = self._open
        e1 = torch.cuda.Event(enable_timing=True)
        e1.record()
        self.spans.append((kind, work, e0, e1, launches))
        self._open = None

    def summary(self, drop_outliers=False):
        """kind -> (launches, total work, total milliseconds); call after a synchronize.  drop_outliers: a span that took
        more than ten times the median of the spans with the same kind and work (a stall of the host or of the box, not of
        the kernel) is left out, work and time both."""
        times = [(kind, work, e0.elapsed_time(e1), launches) for kind, work, e0, e1, launches in self.spans]
        med = {}
        if drop_outliers:
            groups = {}
            for kind, work, ms, _ in times:
                groups.setdefault((kind, work), []).append(ms)
            med = {k: sorted(v)[len(v) // 2] for k, v in groups.items()}
        out = {}
        for kind, work, ms, launches in times:
            if drop_outliers and ms > 10.0 * med[(kind, work)]:
                continue
            n, w, t = out.get(kind, (0, 0, 0.0))
            out[kind] = (n + launches, w + work, t + ms)
        return out

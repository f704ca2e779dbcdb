"""GPU parity at the full sizes of the benchmark configs, in the launch configuration bench.py times
(the same Block driver classes), on outputs the oracle can compute.

Config 1: the whole chain on its own tensors (abs-max -> scale -> cast -> NT product), everything compared whole.
Configs 4 and 5, one test per linear layer and one per attention:
  casts   -- abs-max, scale, reciprocal scale and EVERY cast byte (plain and transposed) bit-exact against the
             oracle (the oracle's cast is O(n); it is called on row chunks only to bound its temporaries);
  GEMMs   -- a row sample of every product (first and last rows of the matrix and rows spread over every
             256-row tile, all columns, the full contraction) against the float64 oracle; the oracle's operands
             are its OWN cast bytes (which the step above proved equal to the library's);
  attention -- four (batch, head) pairs in full (first, last, two seeded), forward and backward.
Configs 2 and 3 are covered whole in test_gpu_gemm.py and test_gpu_attention.py.
"""
import sys

import numpy as np
import pytest
import torch

from oracle import attention, bf16, fp8, gemm, scaling
from paper_2505_20524_amd import block, fog, synth
import mfma_model
from parity import check_attention, check_bf16, check_gemm_elementwise, dev, fscalar, host_u16

pytestmark = pytest.mark.gpu


def progress(msg):
    """A line on the real stderr (not captured): a long test shows that it is alive."""
    print("[configs] " + msg, file=sys.__stderr__, flush=True)


def sample_rows(n, per_tile=1, tile=256, seed=0):
    rng = np.random.default_rng(seed)
    rows = {0, 1, n - 2, n - 1}
    for t0 in range(0, n, tile):
        for _ in range(per_tile):
            rows.add(int(min(n - 1, t0 + rng.integers(tile))))
    return np.array(sorted(rows))


def oracle_cast_whole(bits, fmt, chunk_elems=1 << 22):
    """The oracle's abs-max, scale and cast of a whole 2-D tensor; the cast is evaluated on row chunks."""
    a = scaling.amax(bits)
    rho, rinv = scaling.compute_scale(a, fmt)
    rows_per = max(1, chunk_elems // bits.shape[1])
    q = np.empty(bits.shape, np.uint8)
    for r0 in range(0, bits.shape[0], rows_per):
        q[r0:r0 + rows_per] = scaling.quantize(bits[r0:r0 + rows_per], rho, fmt)
    return a, rho, rinv, q


def check_cast_whole(c, bits, fmt, what):
    a, rho, rinv, want = oracle_cast_whole(bits, fmt)
    assert np.float32(c.amax.item()) == a, what
    assert np.float32(c.scale.item()) == rho and np.float32(c.sinv.item()) == rinv, what
    got = c.q.cpu().numpy()
    assert np.array_equal(got, want), "%s: %d cast bytes differ" % (what, int((got != want).sum()))
    if c.qT is not None:
        assert np.array_equal(c.qT.cpu().numpy(), want.T), what + " (transposed copy)"
    return want, rinv


LINEARS = [(cid, idx) for cid in (5, 4) for idx in range(len(synth.CONFIGS[cid].linears))]


@pytest.mark.parametrize("cid,idx", LINEARS)
def test_config_linear_layer(cid, idx):
    cfg = synth.CONFIGS[cid]
    lin = cfg.linears[idx]
    progress("config %d %s: generating %dx%dx%d" % (cid, lin.name, lin.M, lin.N, lin.K))
    t = synth.linear_tensors(cfg, idx)
    # the first linear in the arrangement with transposed copies (fused cast + transpose, NT weight gradient),
    # the others as the benchmark runs them (row-major casts, TN weight gradient): both at full size
    step = block.LinearStep(lin, t, transposed_wgrad=(idx == 0))
    step.run()
    torch.cuda.synchronize()
    progress("config %d %s: casts whole" % (cid, lin.name))
    Xq, xinv = check_cast_whole(step.X, t["X"], fp8.E4M3, "cfg%d %s X" % (cid, lin.name))
    Wq, winv = check_cast_whole(step.W, t["W"], fp8.E4M3, "cfg%d %s W" % (cid, lin.name))
    dYq, ginv = check_cast_whole(step.dY, t["dY"], fp8.E5M2, "cfg%d %s dY" % (cid, lin.name))
    Y, dX, dW = host_u16(step.Y), host_u16(step.dX), host_u16(step.dW)
    rm = sample_rows(lin.M, seed=idx)
    rn = sample_rows(lin.N, seed=100 + idx)
    progress("config %d %s: GEMM rows" % (cid, lin.name))
    ref = gemm.fp8_gemm_rows(gemm.NT, Xq, fp8.E4M3, xinv, Wq, fp8.E4M3, winv, rm)          # Y = X W^T
    check_bf16(Y[rm], ref, what="cfg%d %s fwd" % (cid, lin.name))
    ref = gemm.fp8_gemm_rows(gemm.NN, dYq, fp8.E5M2, ginv, Wq, fp8.E4M3, winv, rm)         # dX = dY W
    check_bf16(dX[rm], ref, what="cfg%d %s dgrad" % (cid, lin.name))
    ref = gemm.fp8_gemm_rows(gemm.TN, dYq, fp8.E5M2, ginv, Xq, fp8.E4M3, xinv, rn)         # dW = dY^T X
    check_bf16(dW[rn], ref, what="cfg%d %s wgrad" % (cid, lin.name))
    del step
    torch.cuda.empty_cache()


def four_heads(a, seed):
    """First, last and two seeded (batch, head) pairs, distinct."""
    rng = np.random.default_rng(seed)
    heads = [(0, 0), (a.B - 1, a.H - 1)]
    while len(heads) < min(4, a.B * a.H):
        bh = (int(rng.integers(a.B)), int(rng.integers(a.H)))
        if bh not in heads:
            heads.append(bh)
    return heads


@pytest.mark.parametrize("cid", [5, 4])
def test_config_attention(cid):
    cfg = synth.CONFIGS[cid]
    a = cfg.attn
    progress("config %d attention: generating" % cid)
    t = synth.attention_tensors(cfg)
    att = block.AttentionStep(a, t)
    att.run()                               # first pass calibrates the delayed scale of dS
    rho = att.scale_ds.clone()              # the scale the second pass uses
    att.run()
    torch.cuda.synchronize()
    progress("config %d attention: casts whole" % cid)
    c = {}
    for name, fmt in (("Q", fp8.E4M3), ("K", fp8.E4M3), ("V", fp8.E4M3), ("dO", fp8.E5M2)):
        q, rinv = check_cast_whole(att.c[name], t[name].reshape(-1, a.D), fmt, "cfg%d %s" % (cid, name))
        c[name] = (q.reshape(a.B, a.H, a.S, a.D), rinv)
    O = host_u16(att.O).reshape(a.B, a.H, a.S, a.D)
    lse = att.lse.cpu().numpy().reshape(a.B, a.H, a.S)
    assert np.isfinite(lse).all() and np.isfinite(bf16.bits_to_f64(O)).all()
    s = att.s
    rho_ds = np.float32(rho.item())
    dQ, dK, dV = (host_u16(x).reshape(a.B, a.H, a.S, a.D) for x in (att.dQ, att.dK, att.dV))
    do_bits = t["dO"]
    amax_seen = 0.0
    for (b, h) in four_heads(a, cid):
        progress("config %d attention: head (%d, %d)" % (cid, b, h))
        args = (c["Q"][0][b, h], c["K"][0][b, h], c["V"][0][b, h], c["Q"][1], c["K"][1], c["V"][1])
        Or, lr, _ = attention.attn_fwd_head(*args, s, 448.0, True)
        dx = mfma_model.logit_uncertainty(args[0], args[1], args[3], args[4], s, True)
        slack = mfma_model.fwd_cast_slack(*args, s, 448.0, True, dx=dx)
        check_attention(O[b, h], Or, slack, what="cfg%d O[%d,%d]" % (cid, b, h))
        assert np.all(np.abs(lse[b, h] - lr) <= 2e-4 + mfma_model.lse_uncertainty(args[0], args[1], args[3], args[4], s, True, dx=dx))
        # Backward: the GPU consumed its OWN forward results (end-to-end flow of the benchmark).  Exactly those
        # O / lse bits go to the oracle, with the scale of dS the kernel used.
        bargs = args + (O[b, h], do_bits[b, h], c["dO"][0][b, h], c["dO"][1], lse[b, h], s, 448.0, rho_ds, True)
        r = attention.attn_bwd_head(*bargs)
        sl = mfma_model.bwd_cast_slack(*bargs, dx=dx)
        check_attention(dQ[b, h], r[0], sl[0], what="cfg%d dQ[%d,%d]" % (cid, b, h))
        check_attention(dK[b, h], r[1], sl[1], what="cfg%d dK[%d,%d]" % (cid, b, h))
        check_attention(dV[b, h], r[2], sl[2], what="cfg%d dV[%d,%d]" % (cid, b, h))
        amax_seen = max(amax_seen, float(r[3]))
    assert att.amax_ds.item() >= amax_seen * (1 - 1e-4)      # the kernel's abs-max covers every head


def test_config1_end_to_end_on_its_own_tensors():
    """Config 1 (X 512 x 1024 with four x50 outlier channels, W 1024 x 1024): abs-max -> scale -> cast -> NT
    product, every intermediate compared whole: bit-exact scalars and bytes, Y inside the gate.  Run twice,
    through the one-call just-in-time cast and through the three separate calls."""
    cfg = synth.CONFIGS[1]
    lin = cfg.linears[0]
    t = synth.linear_tensors(cfg, 0, want=("X", "W"))
    ora = {}
    for name in ("X", "W"):
        a = scaling.amax(t[name])
        rho, rinv = scaling.compute_scale(a, fp8.E4M3)
        ora[name] = (scaling.quantize(t[name], rho, fp8.E4M3), a, rho, rinv)
    ref = gemm.fp8_gemm(gemm.NT, ora["X"][0], fp8.E4M3, ora["X"][3], ora["W"][0], fp8.E4M3, ora["W"][3])
    for route in ("jit", "separate"):
        casts = {name: block.Cast(dev(t[name]), fog.E4M3, transpose=False) for name in ("X", "W")}
        for name, cst in casts.items():
            cst.run() if route == "jit" else cst.run_separate()
        Y = torch.full((lin.M, lin.N), 0x7FC0, dtype=torch.int16, device="cuda")
        fog.fp8_gemm(fog.NT, lin.M, lin.N, lin.K, casts["X"].q, fog.E4M3, casts["X"].sinv, casts["W"].q, fog.E4M3, casts["W"].sinv, Y)
        torch.cuda.synchronize()
        for name, cst in casts.items():
            want, a, rho, rinv = ora[name]
            assert np.float32(cst.amax.item()) == a and np.float32(cst.scale.item()) == rho and np.float32(cst.sinv.item()) == rinv
            assert np.array_equal(cst.q.cpu().numpy(), want), "%s bytes (%s)" % (name, route)
        stats = check_bf16(host_u16(Y), ref, what="config 1 Y (%s)" % route)
        assert stats["max_steps"] <= 1
        mag = np.float64(ora["X"][3]) * np.float64(ora["W"][3]) * (np.abs(fp8.decode(ora["X"][0], fp8.E4M3)) @ np.abs(fp8.decode(ora["W"][0], fp8.E4M3)).T)
        check_gemm_elementwise(host_u16(Y), ref, mag, what="config 1 Y (%s)" % route)

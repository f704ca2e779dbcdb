"""GPU parity: FP8 attention forward / backward against the float64 oracle."""
import math

import numpy as np
import pytest
import torch

from oracle import attention, bf16, fp8, scaling
from paper_2505_20524_amd import fog, synth
import mfma_model
from parity import check_attention, check_bf16, dev, fscalar, host_u16

pytestmark = pytest.mark.gpu

SAMPLED_EXCEED = 0.06     # a sample of 18 rows, a third of them short (0, 1, 63, 64, ...): one short row may move whole (measured: none did)


def cast_all(q, k, v, do):
    out = {}
    for name, t, fmt in (("q", q, fp8.E4M3), ("k", k, fp8.E4M3), ("v", v, fp8.E4M3), ("do", do, fp8.E5M2)):
        rho, rinv = scaling.compute_scale(scaling.amax(t), fmt)
        out[name] = (scaling.quantize(t.reshape(-1, t.shape[-1]), rho, fmt).reshape(t.shape), rinv)
    return out


def kv_of(c, h):
    """Key/value head of query head h: the tensors of c["k"], c["v"] are [B, H_kv, S, D] (H_kv == H: multi-head)."""
    H, Hkv = c["q"][0].shape[1], c["k"][0].shape[1]
    return h // (H // Hkv)


def gpu_fwd(c, B, H, S, s, causal, want_amax=True, rho_p=448.0):
    O = torch.full((B, H, S, 128), 0x7FC0, dtype=torch.int16, device="cuda")
    lse = torch.full((B, H, S), float("nan"), device="cuda")
    am = torch.full((1,), -1.0, device="cuda") if want_amax else None
    fog.fp8_attn_fwd(B, H, S, 128, s, causal, dev(c["q"][0]), dev(c["k"][0]), dev(c["v"][0]),
                     fscalar(c["q"][1]), fscalar(c["k"][1]), fscalar(c["v"][1]), fscalar(rho_p), O, lse, amax_p=am,
                     H_kv=c["k"][0].shape[1])
    torch.cuda.synchronize()
    return host_u16(O), lse.cpu().numpy(), (am.item() if want_amax else None)


def oracle_fwd_heads(c, heads, s, causal, rho_p=448.0):
    res = {}
    for (b, h) in heads:
        hk = kv_of(c, h)
        res[(b, h)] = attention.attn_fwd_head(c["q"][0][b, h], c["k"][0][b, hk], c["v"][0][b, hk],
                                              c["q"][1], c["k"][1], c["v"][1], s, rho_p, causal)
    return res


def check_fwd(c, B, H, S, s, causal, heads, rho_p=448.0):
    O, lse, am = gpu_fwd(c, B, H, S, s, causal, rho_p=rho_p)
    rho_p = min(rho_p, 448.0)            # the forward uses a probability scale above the format's maximum as 448
    ref = oracle_fwd_heads(c, heads, s, causal, rho_p)
    pmax = 0.0
    for (b, h), (Or, lr, ap) in ref.items():
        hk = kv_of(c, h)
        dx = mfma_model.logit_uncertainty(c["q"][0][b, h], c["k"][0][b, hk], c["q"][1], c["k"][1], s, causal)
        slack = mfma_model.fwd_cast_slack(c["q"][0][b, h], c["k"][0][b, hk], c["v"][0][b, hk], c["q"][1], c["k"][1], c["v"][1],
                                         s, rho_p, causal, dx=dx)
        check_attention(O[b, h], Or, slack, what="O[%d,%d]" % (b, h))
        lunc = mfma_model.lse_uncertainty(c["q"][0][b, h], c["k"][0][b, hk], c["q"][1], c["k"][1], s, causal, dx=dx)
        assert np.all(np.abs(lse[b, h] - lr) <= 2e-4 + lunc), "lse"
        pmax = max(pmax, float(ap))
    assert np.isfinite(lse).all()
    if len(heads) == B * H:
        assert abs(am - pmax) <= 1e-4 * pmax
    assert 0.5 < am <= 1.0 + 1e-6
    return O, lse


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("B,H,S", [(1, 1, 64), (1, 2, 128), (2, 2, 320), (1, 3, 576)])
def test_forward_parity(B, H, S, causal):
    q, k, v, do = synth.small_attention(1000 + S, B, H, S)
    c = cast_all(q, k, v, do)
    check_fwd(c, B, H, S, 1 / math.sqrt(128), causal, [(b, h) for b in range(B) for h in range(H)])


@pytest.mark.parametrize("rho_p", [100.0, 1000.0, 3000.0])
def test_probability_scale_other_than_the_format_maximum(rho_p):
    """scale_p below 448 wastes range.  Above 448 the forward uses 448 (p is taken against the running row reference
    there, so saturation would depend on the visiting order); the backward casts the normalised P, for which
    saturation is well defined (P > 448 / scale_p maps to 448), and takes its saturating-cast loops."""
    B, H, S = 1, 2, 256
    q, k, v, do = synth.small_attention(500 + int(rho_p), B, H, S)
    c = cast_all(q, k, v, do)
    heads = [(0, 0), (0, 1)]
    check_fwd(c, B, H, S, 0.125, True, heads, rho_p=rho_p)
    run_bwd(c, B, H, S, 0.125, True, heads, do, rho_p=rho_p)


def test_forward_fog_softmax_scale_and_q_zero():
    B, H, S = 1, 2, 256
    q, k, v, do = synth.small_attention(77, B, H, S)
    c = cast_all(q, k, v, do)
    check_fwd(c, B, H, S, 0.125, True, [(0, 0), (0, 1)])         # FOG's s = gamma_0^2 / sqrt(D) at D = 128
    # Q = 0: every p is 1 and P~ = 448 exactly, so O_i is the running mean of the decoded V rows
    c["q"] = (np.zeros_like(c["q"][0]), np.float32(1.0))
    O, lse, _ = gpu_fwd(c, B, H, S, 0.125, True)
    for h in range(H):
        vv = fp8.decode(c["v"][0][0, h], fp8.E4M3) * np.float64(c["v"][1])
        run = np.cumsum(vv, axis=0) / np.arange(1, S + 1)[:, None]
        check_bf16(O[0, h], run, rel=1e-5, what="running mean")
        assert np.abs(lse[0, h] - np.log2(np.arange(1, S + 1))).max() < 1e-5


def run_bwd(c, B, H, S, s, causal, heads, do_bits, rho_p=448.0, ds_scale_factor=1.0):
    """Feeds the ORACLE's forward results (O rounded to bf16, lse rounded to binary32) to both sides.
    Under grouped-query attention dK and dV of a key/value head are checked when all the query heads of
    its group are in `heads`: the oracle's per-head contributions are summed in float64 (the kernel sums
    them in binary32 before its one rounding), and so are the slacks of the cast decisions."""
    Hkv = c["k"][0].shape[1]
    G = H // Hkv
    O_bits = np.zeros((B, H, S, 128), np.uint16)
    lse = np.zeros((B, H, S), np.float32)

    def head_args(b, h):
        hk = h // G
        return (c["q"][0][b, h], c["k"][0][b, hk], c["v"][0][b, hk], c["q"][1], c["k"][1], c["v"][1])

    for (b, h) in heads:
        Or, lr, _ = attention.attn_fwd_head(*head_args(b, h), s, rho_p, causal)
        O_bits[b, h] = bf16.f64_to_bits_rne(Or)
        lse[b, h] = lr.astype(np.float32)
    # calibrate rho_dS from one oracle pass without the dS cast (delayed-style scale)
    amax_ds = 0.0
    for (b, h) in heads:
        r = attention.attn_bwd_head(*head_args(b, h), O_bits[b, h], do_bits[b, h], c["do"][0][b, h], c["do"][1], lse[b, h],
                                    s, rho_p, 1.0, causal, True, False)
        amax_ds = max(amax_ds, float(r[3]))
    rho_ds, _ = scaling.compute_scale(np.float32(amax_ds), fp8.E5M2)
    rho_ds = np.float32(rho_ds * ds_scale_factor)     # > 1: a stale (delayed) scale, the largest dS saturate
    dQ = torch.full((B, H, S, 128), 0x7FC0, dtype=torch.int16, device="cuda")
    dK, dV = (torch.full((B, Hkv, S, 128), 0x7FC0, dtype=torch.int16, device="cuda") for _ in range(2))
    am = torch.full((1,), -1.0, device="cuda")
    ws = torch.empty(fog.fp8_attn_workspace(B, H, S, 128, True, H_kv=Hkv), dtype=torch.uint8, device="cuda")
    fog.fp8_attn_bwd(B, H, S, 128, s, causal, dev(c["q"][0]), dev(c["k"][0]), dev(c["v"][0]),
                     fscalar(c["q"][1]), fscalar(c["k"][1]), fscalar(c["v"][1]), dev(O_bits), dev(do_bits), dev(c["do"][0]),
                     fscalar(c["do"][1]), dev(lse), fscalar(rho_p), fscalar(rho_ds), dQ, dK, dV, amax_ds=am, workspace=ws,
                     H_kv=Hkv)
    torch.cuda.synchronize()
    dQ, dK, dV = host_u16(dQ), host_u16(dK), host_u16(dV)
    group = {}
    for (b, h) in heads:
        tail = (O_bits[b, h], do_bits[b, h], c["do"][0][b, h], c["do"][1], lse[b, h], s, rho_p, rho_ds, causal)
        r = attention.attn_bwd_head(*head_args(b, h), *tail)
        sl = mfma_model.bwd_cast_slack(*head_args(b, h), *tail)
        check_attention(dQ[b, h], r[0], sl[0], what="dQ[%d,%d]" % (b, h))
        acc = group.setdefault((b, h // G), [0, 0.0, 0.0, 0.0, 0.0])
        acc[0] += 1
        acc[1] = acc[1] + r[1]; acc[2] = acc[2] + r[2]; acc[3] = acc[3] + sl[1]; acc[4] = acc[4] + sl[2]
    checked = 0
    for (b, hk), (n, dk, dv, sk, sv) in group.items():
        if n != G:
            continue            # not every query head of the group was evaluated
        check_attention(dK[b, hk], dk, sk, what="dK[%d,%d]" % (b, hk))
        check_attention(dV[b, hk], dv, sv, what="dV[%d,%d]" % (b, hk))
        checked += 1
    assert checked > 0
    if len(heads) == B * H:
        assert abs(am.item() - amax_ds) <= 1e-4 * amax_ds
    return dQ, dK, dV


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("B,H,S", [(1, 1, 64), (1, 2, 128), (2, 2, 320), (1, 2, 576)])
def test_backward_parity(B, H, S, causal):
    q, k, v, do = synth.small_attention(2000 + S, B, H, S)
    c = cast_all(q, k, v, do)
    run_bwd(c, B, H, S, 1 / math.sqrt(128), causal, [(b, h) for b in range(B) for h in range(H)], do)


@pytest.mark.parametrize("factor", [4.0, 64.0])
def test_backward_with_a_stale_ds_scale_saturates_like_the_oracle(factor):
    """A scale of dS several times too large (delayed scaling after the gradients grew): rho_ds dS exceeds the largest
    finite E5M2 value in some key blocks and not in others, so both the clamped and the unclamped form of the cast run."""
    B, H, S = 1, 2, 320
    q, k, v, do = synth.small_attention(2600 + int(factor), B, H, S)
    c = cast_all(q, k, v, do)
    run_bwd(c, B, H, S, 1 / math.sqrt(128), True, [(b, h) for b in range(B) for h in range(H)], do, ds_scale_factor=factor)


def gqa_case(seed, B, H, Hkv, S):
    """Grouped-query inputs: Q and dO with H heads, K and V with H_kv heads (same recipe, own seed)."""
    q, _, _, do = synth.small_attention(seed, B, H, S)
    _, k, v, _ = synth.small_attention(seed + 1, B, Hkv, S)
    return cast_all(q, k, v, do), do


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("B,H,Hkv,S", [(1, 2, 1, 128), (2, 4, 2, 320), (1, 8, 2, 192), (1, 4, 1, 448)])
def test_grouped_query_parity(B, H, Hkv, S, causal):
    """H_kv < H (Appendix B: grouped-query attention): forward per query head against its group's K/V,
    backward with dK/dV summed over the group."""
    c, do = gqa_case(3000 + S + H, B, H, Hkv, S)
    heads = [(b, h) for b in range(B) for h in range(H)]
    check_fwd(c, B, H, S, 1 / math.sqrt(128), causal, heads)
    run_bwd(c, B, H, S, 1 / math.sqrt(128), causal, heads, do)


@pytest.mark.parametrize("B,H,Hkv,S", [(2, 4, 2, 8192), (1, 2, 1, 16384)])
def test_long_context_grouped_query_sampled(B, H, Hkv, S):
    """Sequences of 8192 and 16384 tokens with grouped queries, causal, whole on the GPU; the oracle
    evaluates sampled outputs one by one.  Under the causal mask row i of O / lse / dQ depends on the
    keys 0..i only, and row j of dK / dV on the queries j..S-1 only, so each sample is the oracle's own
    (unmasked) routine on that slice of the head: no S x S matrix is ever formed.  The backward pass
    consumes the GPU's own forward results on both sides, as a training step does."""
    G = H // Hkv
    c, do = gqa_case(S + H, B, H, Hkv, S)
    s = 0.125
    O, lse, _ = gpu_fwd(c, B, H, S, s, True)
    assert np.isfinite(lse).all()
    rng = np.random.default_rng(S)
    rows = sorted({0, 1, 63, 64, 127, 128, S // 2 - 1, S // 2, S - 65, S - 64, S - 2, S - 1, *map(int, rng.integers(0, S, 6))})
    heads = [(0, 0), (B - 1, H - 1)]
    sq, sk, sv = c["q"][1], c["k"][1], c["v"][1]
    for (b, h) in heads:
        hk = h // G
        refs, slacks = [], []
        for i in rows:
            args = (c["q"][0][b, h, i:i + 1], c["k"][0][b, hk, :i + 1], c["v"][0][b, hk, :i + 1], sq, sk, sv)
            Or, lr, _ = attention.attn_fwd_head(*args, s, 448.0, False)
            dx = mfma_model.logit_uncertainty(args[0], args[1], sq, sk, s, False)
            refs.append(Or)
            slacks.append(mfma_model.fwd_cast_slack(*args, s, 448.0, False, dx=dx))
            lunc = mfma_model.lse_uncertainty(args[0], args[1], sq, sk, s, False, dx=dx)
            assert np.all(np.abs(lse[b, h, i:i + 1] - lr) <= 2e-4 + lunc)
        # the sampled rows of a head as one tensor; a third of them are short rows (0, 1, 63, 64, ...), where a
        # single two-code element of P moves the whole row
        check_attention(O[b, h, rows], np.concatenate(refs), np.concatenate(slacks), what="O[%d,%d] rows" % (b, h),
                        max_exceed_frac=SAMPLED_EXCEED)
    # backward on the GPU's own O and lse; the scale of dS from a first pass (delayed-style)
    Od, lsed = dev(O), dev(lse)
    dQ = torch.full((B, H, S, 128), 0x7FC0, dtype=torch.int16, device="cuda")
    dK, dV = (torch.full((B, Hkv, S, 128), 0x7FC0, dtype=torch.int16, device="cuda") for _ in range(2))
    am = torch.full((1,), -1.0, device="cuda")
    ws = torch.empty(fog.fp8_attn_workspace(B, H, S, 128, True, H_kv=Hkv), dtype=torch.uint8, device="cuda")
    dev_in = (dev(c["q"][0]), dev(c["k"][0]), dev(c["v"][0]), fscalar(sq), fscalar(sk), fscalar(sv), Od, dev(do), dev(c["do"][0]),
              fscalar(c["do"][1]), lsed, fscalar(448.0))
    fog.fp8_attn_bwd(B, H, S, 128, s, True, *dev_in, fscalar(1.0), dQ, dK, dV, amax_ds=am, workspace=ws, H_kv=Hkv)
    torch.cuda.synchronize()
    rho_ds, _ = scaling.compute_scale(np.float32(am.item()), fp8.E5M2)
    fog.fp8_attn_bwd(B, H, S, 128, s, True, *dev_in, fscalar(rho_ds), dQ, dK, dV, amax_ds=am, workspace=ws, H_kv=Hkv)
    torch.cuda.synchronize()
    dQ, dK, dV = host_u16(dQ), host_u16(dK), host_u16(dV)
    sdo = c["do"][1]

    def bwd_slice(b, h, qs, ks):
        """Oracle backward of query head (b, h) restricted to queries qs and keys ks (all visible)."""
        hk = h // G
        args = (c["q"][0][b, h, qs], c["k"][0][b, hk, ks], c["v"][0][b, hk, ks], sq, sk, sv,
                O[b, h, qs], do[b, h, qs], c["do"][0][b, h, qs], sdo, lse[b, h, qs], s, 448.0, rho_ds, False)
        return attention.attn_bwd_head(*args), mfma_model.bwd_cast_slack(*args)

    for (b, h) in heads:
        res = [bwd_slice(b, h, slice(i, i + 1), slice(0, i + 1)) for i in rows]
        check_attention(dQ[b, h, rows], np.concatenate([r[0] for r, _ in res]), np.concatenate([sl[0] for _, sl in res]),
                        what="dQ[%d,%d] rows" % (b, h), max_exceed_frac=SAMPLED_EXCEED)
    for (b, hk) in [(0, 0), (B - 1, Hkv - 1)]:
        dks, dvs, slks, slvs = [], [], [], []
        for j in rows:
            dk = dv = slk = slv = 0.0
            for h in range(hk * G, hk * G + G):            # the group's query heads all feed this key
                r, sl = bwd_slice(b, h, slice(j, S), slice(j, j + 1))
                dk, dv, slk, slv = dk + r[1], dv + r[2], slk + sl[1], slv + sl[2]
            dks.append(dk); dvs.append(dv); slks.append(slk); slvs.append(slv)
        check_attention(dK[b, hk, rows], np.concatenate(dks), np.concatenate(slks), what="dK[%d,%d] rows" % (b, hk),
                        max_exceed_frac=SAMPLED_EXCEED)
        check_attention(dV[b, hk, rows], np.concatenate(dvs), np.concatenate(slvs), what="dV[%d,%d] rows" % (b, hk),
                        max_exceed_frac=SAMPLED_EXCEED)


def test_backward_two_launch_form_noncausal():
    """Enough key blocks (B H_kv S / 128 >= 1024) for dK and dV to be produced by two launches instead of
    one; non-causal, two heads checked in full (config 3 below covers the causal case of that form)."""
    B, H, S = 8, 16, 1024
    q, k, v, do = synth.small_attention(4242, B, H, S)
    c = cast_all(q, k, v, do)
    run_bwd(c, B, H, S, 1 / math.sqrt(128), False, [(0, 0), (B - 1, H - 1)], do)


def test_config3_full_size_sampled_heads():
    """Config 3 whole on the GPU (B 4, H 16, S 2048, D 128, causal); the oracle checks 4 (batch, head)
    pairs in full (first, last, two seeded), forward and backward; every head is checked for sanity."""
    cfg = synth.CONFIGS[3]
    a = cfg.attn
    t = synth.attention_tensors(cfg)
    c = cast_all(t["Q"], t["K"], t["V"], t["dO"])
    rng = np.random.default_rng(3)
    heads = [(0, 0), (a.B - 1, a.H - 1)]
    while len(heads) < 4:
        bh = (int(rng.integers(a.B)), int(rng.integers(a.H)))
        if bh not in heads:
            heads.append(bh)
    s = 1 / math.sqrt(128)
    O, lse = check_fwd(c, a.B, a.H, a.S, s, True, heads)
    Of = bf16.bits_to_f64(O)
    assert np.isfinite(Of).all()
    # every output row is a convex combination of decoded V rows (up to the cast of P): bounded by max |V|
    vmax = np.abs(fp8.decode(c["v"][0], fp8.E4M3)).max() * float(c["v"][1])
    assert np.abs(Of).max() <= vmax * 1.07
    run_bwd(c, a.B, a.H, a.S, s, True, heads, t["dO"])


def test_optional_abs_max_outputs_may_be_null():
    """amax_p and amax_ds are optional: without them the kernels take the instantiations that skip the
    running maxima, and the results are bit-identical to the calls that report them."""
    B, H, S = 1, 2, 192
    q, k, v, do = synth.small_attention(909, B, H, S)
    c = cast_all(q, k, v, do)
    s = 0.125
    O1, lse1, _ = gpu_fwd(c, B, H, S, s, True, want_amax=True)
    O2, lse2, _ = gpu_fwd(c, B, H, S, s, True, want_amax=False)
    assert np.array_equal(O1, O2) and np.array_equal(lse1, lse2)
    res = []
    for with_amax in (True, False):
        dQ, dK, dV = (torch.full((B, H, S, 128), 0x7FC0, dtype=torch.int16, device="cuda") for _ in range(3))
        am = torch.zeros(1, device="cuda") if with_amax else None
        ws = torch.empty(fog.fp8_attn_workspace(B, H, S, 128, True), dtype=torch.uint8, device="cuda")
        fog.fp8_attn_bwd(B, H, S, 128, s, True, dev(c["q"][0]), dev(c["k"][0]), dev(c["v"][0]), fscalar(c["q"][1]), fscalar(c["k"][1]),
                         fscalar(c["v"][1]), dev(O1), dev(do), dev(c["do"][0]), fscalar(c["do"][1]), dev(lse1), fscalar(448.0),
                         fscalar(2.0 ** 20), dQ, dK, dV, amax_ds=am, workspace=ws)
        torch.cuda.synchronize()
        res.append([host_u16(x) for x in (dQ, dK, dV)])
    assert all(np.array_equal(a, b) for a, b in zip(*res))


def test_attention_argument_errors():
    lib = fog.load()
    st = torch.cuda.current_stream().cuda_stream
    x = torch.zeros(64 * 128, dtype=torch.uint8, device="cuda")
    o = torch.zeros(64 * 128, dtype=torch.int16, device="cuda")
    f = fscalar(1.0)
    l = torch.zeros(64, device="cuda")
    p, fp = x.data_ptr(), f.data_ptr()
    args = lambda D, S, q=p, H=1, Hkv=1: (1, H, Hkv, S, D, 0.1, 1, q, p, p, fp, fp, fp, fp, o.data_ptr(), l.data_ptr(), None, None, 0, st)
    assert lib.fog_fp8_attn_fwd(*args(64, 64)) == 4
    assert lib.fog_fp8_attn_fwd(*args(128, 48)) == 4
    assert lib.fog_fp8_attn_fwd(*args(128, 64, None)) == 1
    assert lib.fog_fp8_attn_fwd(*args(128, 64, p + 4)) == 3
    assert lib.fog_fp8_attn_fwd(*args(128, 64)) == 0
    assert lib.fog_fp8_attn_fwd(*args(128, 64, p, 3, 2)) == 2          # H not a multiple of H_kv
    assert lib.fog_fp8_attn_fwd(*args(128, 64, p, 2, 0)) == 2
    b = (1, 1, 1, 64, 128, 0.1, 1, p, p, p, fp, fp, fp, o.data_ptr(), o.data_ptr(), p, fp, l.data_ptr(), fp, fp,
         o.data_ptr(), o.data_ptr(), o.data_ptr(), None)
    assert lib.fog_fp8_attn_bwd(*b, None, 0, st) == 5
    ws = torch.zeros(3 * 64, device="cuda")
    assert lib.fog_fp8_attn_bwd(*b, ws.data_ptr(), 100, st) == 5
    assert lib.fog_fp8_attn_bwd(*b, ws.data_ptr(), 3 * 64 * 4, st) == 0
    torch.cuda.synchronize()


def test_forward_with_integer_logits_has_no_open_decision():
    """Inputs built so that every logit is a small integer in the log2 domain: every p is a power of two, whose
    E4M3 cast is the same whichever side evaluates it (powers of two sit far from rounding boundaries), so no
    slack is granted: O must meet the plain gate, lse a tight one.  Q~ rows are one-hot (1 or 2 at column
    i mod 128), K~ holds integers -3..3, both scales are 1 and s = ln 2, so x_ij = q_i k_j,(i mod 128)."""
    B, H, S = 1, 2, 320
    rng = np.random.default_rng(99)
    Q8 = np.zeros((B, H, S, 128), np.uint8)
    one, two = int(fp8.encode_sat(np.float32(1.0), fp8.E4M3)), int(fp8.encode_sat(np.float32(2.0), fp8.E4M3))
    for h in range(H):
        for i in range(S):
            Q8[0, h, i, i % 128] = one if rng.random() < 0.5 else two
    K8 = fp8.encode_sat(rng.integers(-3, 4, size=(B, H, S, 128)).astype(np.float32), fp8.E4M3)
    _, _, v, _ = synth.small_attention(98, B, H, S)
    rho_v, vinv = scaling.compute_scale(scaling.amax(v), fp8.E4M3)
    V8 = scaling.quantize(v.reshape(-1, 128), rho_v, fp8.E4M3).reshape(v.shape)
    c = {"q": (Q8, np.float32(1.0)), "k": (K8, np.float32(1.0)), "v": (V8, vinv)}
    s = float(np.float32(np.log(2.0)))
    for causal in (True, False):
        O, lse, am = gpu_fwd(c, B, H, S, s, causal)
        for h in range(H):
            x = attention.logits(Q8[0, h], K8[0, h], 1.0, 1.0, s, causal)
            fin = np.isfinite(x)
            assert np.abs(x[fin] - np.rint(x[fin])).max() < 1e-6 and np.ptp(x[fin]) >= 8      # integers, spread over many binades
            Or, lr, _ = attention.attn_fwd_head(Q8[0, h], K8[0, h], V8[0, h], 1.0, 1.0, vinv, s, 448.0, causal)
            st = check_bf16(O[0, h], Or, what="O, integer logits", max_flip_frac=0.1)
            assert st["max_steps"] <= 1
            assert np.abs(lse[0, h] - lr).max() < 2e-5


def test_backward_with_q_zero_closed_forms():
    """Q~ = 0: every logit is 0, P_ij = 1 / (i + 1) exactly and 448 / (i + 1) never comes near an E4M3 rounding
    boundary for i < 256, so the cast of P is decided alike on both sides: dV must meet the plain gate with no
    slack.  dK = s sinv_q / rho_ds (dS~^T Q~) is a sum of zeros: every element is exactly zero."""
    B, H, S = 1, 2, 256
    q, k, v, do = synth.small_attention(4321, B, H, S)
    c = cast_all(q, k, v, do)
    c["q"] = (np.zeros_like(c["q"][0]), np.float32(1.0))
    s = 0.125
    O_bits = np.zeros((B, H, S, 128), np.uint16)
    lse = np.zeros((B, H, S), np.float32)
    for h in range(H):
        Or, lr, _ = attention.attn_fwd_head(c["q"][0][0, h], c["k"][0][0, h], c["v"][0][0, h], c["q"][1], c["k"][1], c["v"][1], s, 448.0, True)
        O_bits[0, h] = bf16.f64_to_bits_rne(Or)
        lse[0, h] = lr.astype(np.float32)
        assert np.array_equal(lse[0, h], np.log2(np.arange(1, S + 1)).astype(np.float32))
    dQ, dK, dV = (torch.full((B, H, S, 128), 0x7FC0, dtype=torch.int16, device="cuda") for _ in range(3))
    ws = torch.empty(fog.fp8_attn_workspace(B, H, S, 128, True), dtype=torch.uint8, device="cuda")
    rho_ds = np.float32(2.0 ** 16)
    fog.fp8_attn_bwd(B, H, S, 128, s, True, dev(c["q"][0]), dev(c["k"][0]), dev(c["v"][0]), fscalar(c["q"][1]), fscalar(c["k"][1]),
                     fscalar(c["v"][1]), dev(O_bits), dev(do), dev(c["do"][0]), fscalar(c["do"][1]), dev(lse), fscalar(448.0),
                     fscalar(rho_ds), dQ, dK, dV, workspace=ws)
    torch.cuda.synchronize()
    dK, dV = host_u16(dK), host_u16(dV)
    assert np.all((dK & 0x7FFF) == 0)                      # exactly zero (either sign)
    for h in range(H):
        dov = fp8.decode(c["do"][0][0, h], fp8.E5M2) * np.float64(c["do"][1])
        pt = fp8.decode(fp8.encode_sat(np.float32(448.0 / np.arange(1, S + 1)), fp8.E4M3), fp8.E4M3) / 448.0
        want = np.stack([(pt[j:, None] * dov[j:]).sum(0) for j in range(S)])       # dV_j = sum_{i >= j} P~_ij dO_i
        r = attention.attn_bwd_head(c["q"][0][0, h], c["k"][0][0, h], c["v"][0][0, h], c["q"][1], c["k"][1], c["v"][1], O_bits[0, h],
                                    do[0, h], c["do"][0][0, h], c["do"][1], lse[0, h], s, 448.0, rho_ds, True)
        assert np.allclose(r[2], want, rtol=1e-12, atol=1e-18)
        check_bf16(dV[0, h], want, what="dV, Q = 0", max_flip_frac=0.1)


def test_failing_attention_calls_leave_device_memory_untouched():
    """Argument errors are detected before anything is launched: the optional abs-max outputs, which a
    successful call zeroes first, keep their contents when the call fails."""
    lib = fog.load()
    st = torch.cuda.current_stream().cuda_stream
    x = torch.zeros(64 * 128, dtype=torch.uint8, device="cuda")
    o = torch.full((64 * 128,), 0x1234, dtype=torch.int16, device="cuda")
    f = fscalar(1.0)
    l = torch.full((64,), -3.0, device="cuda")
    am = torch.full((1,), -7.0, device="cuda")
    p, fp = x.data_ptr(), f.data_ptr()
    fwd = lambda q, S=64, D=128: lib.fog_fp8_attn_fwd(1, 1, 1, S, D, 0.1, 1, q, p, p, fp, fp, fp, fp, o.data_ptr(), l.data_ptr(),
                                                       am.data_ptr(), None, 0, st)
    assert fwd(None) == 1 and fwd(p + 4) == 3 and fwd(p, S=48) == 4 and fwd(p, D=64) == 4
    bwd = lambda q, ws, wsb: lib.fog_fp8_attn_bwd(1, 1, 1, 64, 128, 0.1, 1, q, p, p, fp, fp, fp, o.data_ptr(), o.data_ptr(), p, fp,
                                                  l.data_ptr(), fp, fp, o.data_ptr(), o.data_ptr(), o.data_ptr(), am.data_ptr(), ws, wsb, st)
    ws = torch.zeros(3 * 64, device="cuda")
    assert bwd(None, ws.data_ptr(), 3 * 64 * 4) == 1 and bwd(p + 4, ws.data_ptr(), 3 * 64 * 4) == 3 and bwd(p, None, 0) == 5
    assert bwd(p, ws.data_ptr(), 100) == 5
    torch.cuda.synchronize()
    assert am.item() == -7.0 and (o == 0x1234).all() and (l == -3.0).all() and (ws == 0).all()
    assert fwd(p) == 0                                   # the same arguments, valid: the call runs and zeroes the abs-max first
    torch.cuda.synchronize()
    assert am.item() != -7.0

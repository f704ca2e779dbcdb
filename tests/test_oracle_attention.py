"""Pins for the oracle's FP8 attention forward / backward (CPU only)."""
import math

import numpy as np
import pytest
import torch

from oracle import attention, bf16, fp8, scaling
from paper_2505_20524_amd import synth


def make_head(seed, S, D=16, do_std=1e-2):
    q, k, v, do = (t[0, 0] for t in synth.small_attention(seed, 1, 1, S, D, do_std))
    out = {}
    for name, t in (("q", q), ("k", k), ("v", v)):
        rho, rinv = scaling.compute_scale(scaling.amax(t), fp8.E4M3)
        out[name] = (scaling.quantize(t, rho, fp8.E4M3), rinv)
    rho, rinv = scaling.compute_scale(scaling.amax(do), fp8.E5M2)
    out["do"] = (scaling.quantize(do, rho, fp8.E5M2), rinv, do)
    return out


def brute_fwd(Q8, K8, V8, sq, sk, sv, s, rho_p, causal):
    """Scalar loops, written from the definition, independent of the vectorised oracle."""
    S, D = Q8.shape
    tab = fp8.decode(np.arange(256, dtype=np.uint8), fp8.E4M3)
    dq = lambda c: float(tab[int(c)])
    O = np.zeros((S, D)); L = np.zeros(S)
    for i in range(S):
        js = range(i + 1) if causal else range(S)
        xs = []
        for j in js:
            acc = 0.0
            for d in range(D):
                acc += dq(Q8[i, d]) * dq(K8[j, d])
            xs.append(s * attention.LOG2E * float(sq) * float(sk) * acc)
        M = math.ceil(max(xs))
        ps = [2.0 ** (x - M) for x in xs]
        l = sum(ps)
        pq = [dq(fp8.encode_sat(np.float32(rho_p * p), fp8.E4M3).item()) for p in ps]
        for d in range(D):
            acc = 0.0
            for jj, j in enumerate(js):
                acc += pq[jj] * dq(V8[j, d])
            O[i, d] = float(sv) * acc / (rho_p * l)
        L[i] = M + math.log2(l)
    return O, L


@pytest.mark.parametrize("causal", [True, False])
def test_forward_vs_brute_force(causal):
    h = make_head(21, 24, 8)
    s = 1 / math.sqrt(8)
    O, lse, amax_p = attention.attn_fwd_head(h["q"][0], h["k"][0], h["v"][0], h["q"][1], h["k"][1], h["v"][1], s, 448.0, causal)
    Ob, Lb = brute_fwd(h["q"][0], h["k"][0], h["v"][0], h["q"][1], h["k"][1], h["v"][1], s, 448.0, causal)
    assert np.allclose(O, Ob, rtol=1e-12, atol=1e-14)
    assert np.allclose(lse, Lb, rtol=1e-13)
    assert 0.5 < amax_p <= 1.0


def test_forward_closed_forms():
    h = make_head(22, 40, 16)
    s = 0.25
    O, lse, _ = attention.attn_fwd_head(h["q"][0], h["k"][0], h["v"][0], h["q"][1], h["k"][1], h["v"][1], s, 448.0, True)
    v = fp8.decode(h["v"][0], fp8.E4M3) * np.float64(h["v"][1])
    # row 0 attends to key 0 only: O_0 = v_0 * decode(cast(448 p)) / (448 p), p = 2^(x_00 - ceil(x_00))
    x00 = s * attention.LOG2E * float(h["q"][1]) * float(h["k"][1]) * float(
        (fp8.decode(h["q"][0][0], fp8.E4M3) * fp8.decode(h["k"][0][0], fp8.E4M3)).sum())
    p00 = 2.0 ** (x00 - math.ceil(x00))
    w = fp8.decode(fp8.encode_sat(np.float32(448.0 * p00), fp8.E4M3), fp8.E4M3).item() / (448.0 * p00)
    assert np.allclose(O[0], v[0] * w, rtol=1e-14, atol=0) and abs(w - 1) <= 2.0 ** -4
    assert abs(lse[0] - x00) < 1e-12
    # Q = 0: every p is 1, P~ = 448 exactly, O_i = running mean of the decoded V rows
    Q0 = np.zeros_like(h["q"][0])
    O0, lse0, _ = attention.attn_fwd_head(Q0, h["k"][0], h["v"][0], 1.0, h["k"][1], h["v"][1], s, 448.0, True)
    run = np.cumsum(v, axis=0) / np.arange(1, 41)[:, None]
    assert np.allclose(O0, run, rtol=1e-14, atol=0)
    assert np.allclose(lse0, np.log2(np.arange(1, 41)), atol=1e-14)


def test_forward_without_p_cast_is_textbook_softmax_attention():
    h = make_head(23, 48, 16)
    s = 0.3
    O, lse, _ = attention.attn_fwd_head(h["q"][0], h["k"][0], h["v"][0], h["q"][1], h["k"][1], h["v"][1], s, 448.0, True, fp8_p=False)
    q = torch.from_numpy(fp8.decode(h["q"][0], fp8.E4M3) * float(h["q"][1]))
    k = torch.from_numpy(fp8.decode(h["k"][0], fp8.E4M3) * float(h["k"][1]))
    v = torch.from_numpy(fp8.decode(h["v"][0], fp8.E4M3) * float(h["v"][1]))
    ref = torch.nn.functional.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True, scale=s)[0].numpy()
    assert np.allclose(O, ref, rtol=1e-11, atol=1e-13)
    lref = torch.logsumexp(s * (q @ k.T) + torch.triu(torch.full((48, 48), -math.inf, dtype=torch.float64), 1), dim=1).numpy() / math.log(2)
    assert np.allclose(lse, lref, rtol=1e-12)
    # with the cast of P on, the result stays within what 3 mantissa bits allow
    O8, _, _ = attention.attn_fwd_head(h["q"][0], h["k"][0], h["v"][0], h["q"][1], h["k"][1], h["v"][1], s, 448.0, True)
    err = np.abs(O8 - O).max() / np.abs(O).max()
    assert 0 < err < 2.0 ** -4


def test_integer_row_reference_commutes_with_the_cast():
    """Shifting the row reference by an integer rescales p by an exact power of two; above the
    subnormal range of E4M3 the cast codes only change exponent, so P~/reference is unchanged."""
    rng = np.random.default_rng(8)
    x = rng.uniform(-6, 0, size=5000)
    for shift in (1, 2, 3):
        t0 = np.float32(448.0 * np.exp2(x))
        t1 = np.float32(448.0 * np.exp2(x - shift))
        c0 = fp8.decode(fp8.encode_sat(t0, fp8.E4M3), fp8.E4M3)
        c1 = fp8.decode(fp8.encode_sat(t1, fp8.E4M3), fp8.E4M3)
        normal = t1 >= 2.0 ** -6
        assert normal.sum() > 4000
        assert np.array_equal(c0[normal], c1[normal] * 2.0 ** shift)


def _bwd_inputs(seed, S, D):
    h = make_head(seed, S, D)
    s = 1 / math.sqrt(D)
    O, lse, _ = attention.attn_fwd_head(h["q"][0], h["k"][0], h["v"][0], h["q"][1], h["k"][1], h["v"][1], s, 448.0, True, fp8_p=False)
    return h, s, O, lse


def test_backward_without_casts_matches_autograd():
    """Casts of P and dS off: the oracle is the textbook softmax-attention gradient, except that
    D_i = rowsum(dO o O) is taken from the bf16 O and dO; that shift has a closed form, removed below."""
    S, D = 20, 8
    h, s, O, lse = _bwd_inputs(31, S, D)
    Ob = bf16.f64_to_bits_rne(O)
    dOb = h["do"][2]
    do_dec = fp8.decode(h["do"][0], fp8.E5M2) * np.float64(h["do"][1])
    q = torch.tensor(fp8.decode(h["q"][0], fp8.E4M3) * float(h["q"][1]), requires_grad=True)
    k = torch.tensor(fp8.decode(h["k"][0], fp8.E4M3) * float(h["k"][1]), requires_grad=True)
    v = torch.tensor(fp8.decode(h["v"][0], fp8.E4M3) * float(h["v"][1]), requires_grad=True)
    go = torch.tensor(do_dec)
    out = torch.nn.functional.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True, scale=s)[0]
    out.backward(go)
    dQ, dK, dV, amax_ds = attention.attn_bwd_head(
        h["q"][0], h["k"][0], h["v"][0], h["q"][1], h["k"][1], h["v"][1], Ob, dOb, h["do"][0], h["do"][1], lse,
        s, 448.0, 1.0, True, fp8_p=False, fp8_ds=False)
    assert np.allclose(dV, v.grad.numpy(), rtol=1e-11, atol=1e-15)          # dV does not involve D
    Dt = (go * out.detach()).sum(1).numpy()                                  # autograd's D
    Do = (bf16.bits_to_f64(dOb) * bf16.bits_to_f64(Ob)).sum(1)               # the oracle's D
    P = torch.softmax(s * (q @ k.T) + torch.triu(torch.full((S, S), -math.inf, dtype=torch.float64), 1), dim=1).detach().numpy()
    corr = -(P * (Do - Dt)[:, None])                                         # dS_oracle - dS_autograd
    assert np.allclose(dQ, q.grad.numpy() + s * corr @ k.detach().numpy(), rtol=1e-9, atol=1e-14)
    assert np.allclose(dK, k.grad.numpy() + s * corr.T @ q.detach().numpy(), rtol=1e-9, atol=1e-14)
    assert np.abs(corr).max() < 0.3 * np.abs(dQ).max() / s                   # the shift is a perturbation, not the signal
    assert amax_ds > 0


def test_backward_formulas_by_finite_differences():
    """FP8 casts off and D computed from exactly representable O, dO: gradients of
    sum(dO o Attn(Q,K,V)) by central differences in float64."""
    S, D = 6, 4
    rng = np.random.default_rng(77)
    # operands on the E4M3 grid so that codes decode exactly; scales 1
    Q8 = rng.integers(0x20, 0x48, size=(S, D), dtype=np.uint8) | (rng.integers(0, 2, size=(S, D), dtype=np.uint8) << 7)
    K8 = rng.integers(0x20, 0x48, size=(S, D), dtype=np.uint8) | (rng.integers(0, 2, size=(S, D), dtype=np.uint8) << 7)
    V8 = rng.integers(0x20, 0x48, size=(S, D), dtype=np.uint8) | (rng.integers(0, 2, size=(S, D), dtype=np.uint8) << 7)
    dO8 = rng.integers(0x30, 0x44, size=(S, D), dtype=np.uint8) | (rng.integers(0, 2, size=(S, D), dtype=np.uint8) << 7)
    s = 0.2
    go = fp8.decode(dO8, fp8.E5M2)
    dOb = bf16.f64_to_bits_rne(go)
    assert np.array_equal(bf16.bits_to_f64(dOb), go)

    def f(q, k, v):
        x = s * q @ k.T + np.triu(np.full((S, S), -np.inf), 1)
        p = np.exp(x - x.max(1, keepdims=True)); p /= p.sum(1, keepdims=True)
        return p @ v

    q0, k0, v0 = (fp8.decode(c, fp8.E4M3) for c in (Q8, K8, V8))
    O = f(q0, k0, v0)
    _, lse, _ = attention.attn_fwd_head(Q8, K8, V8, 1.0, 1.0, 1.0, s, 448.0, True, fp8_p=False)
    # O is not bf16-exact, so D_i from the rounded O carries a shift with a closed form; dV (no D) is checked
    # tightly and dQ/dK against finite differences with that shift removed.
    Ob = bf16.f64_to_bits_rne(O)
    dQ, dK, dV, _ = attention.attn_bwd_head(Q8, K8, V8, 1.0, 1.0, 1.0, Ob, dOb, dO8, 1.0, lse, s, 448.0, 1.0, True, False, False)
    eps = 1e-6

    def num_grad(which):
        g = np.zeros((S, D))
        for i in range(S):
            for d in range(D):
                args = [q0.copy(), k0.copy(), v0.copy()]
                args[which][i, d] += eps
                up = (go * f(*args)).sum()
                args[which][i, d] -= 2 * eps
                dn = (go * f(*args)).sum()
                g[i, d] = (up - dn) / (2 * eps)
        return g

    assert np.allclose(dV, num_grad(2), rtol=1e-7, atol=1e-9)
    x = s * q0 @ k0.T + np.triu(np.full((S, S), -np.inf), 1)
    P = np.exp(x - x.max(1, keepdims=True)); P /= P.sum(1, keepdims=True)
    shift = ((go * bf16.bits_to_f64(Ob)).sum(1) - (go * O).sum(1))
    corr = -(P * shift[:, None])
    assert np.allclose(dQ - s * corr @ k0, num_grad(0), rtol=1e-6, atol=1e-8)
    assert np.allclose(dK - s * corr.T @ q0, num_grad(1), rtol=1e-6, atol=1e-8)


def test_backward_with_casts_stays_within_fp8_error_and_q_zero_closed_form():
    S, D = 32, 16
    h, s, O, lse = _bwd_inputs(33, S, D)
    Ob = bf16.f64_to_bits_rne(O)
    args = (h["q"][0], h["k"][0], h["v"][0], h["q"][1], h["k"][1], h["v"][1], Ob, h["do"][2], h["do"][0], h["do"][1], lse, s, 448.0)
    ref = attention.attn_bwd_head(*args, 1.0, True, False, False)
    rho_ds, _ = scaling.compute_scale(ref[3], fp8.E5M2)
    got = attention.attn_bwd_head(*args, rho_ds, True, True, True)
    for g, r in zip(got[:3], ref[:3]):
        err = np.abs(g - r).max() / np.abs(r).max()
        assert 0 < err < 0.15
    assert got[3] == ref[3]
    # Q = 0 with causal mask: P_ij = 1/(i+1); dV_j = sum_{i>=j} P~_ij dO_i / rho_P with P~ = cast(448/(i+1))
    Q0 = np.zeros_like(h["q"][0])
    lse0 = np.log2(np.arange(1, S + 1, dtype=np.float64))
    dQ, dK, dV, _ = attention.attn_bwd_head(Q0, h["k"][0], h["v"][0], 1.0, h["k"][1], h["v"][1], Ob, h["do"][2], h["do"][0], h["do"][1],
                                            lse0, s, 448.0, rho_ds, True, True, True)
    do = fp8.decode(h["do"][0], fp8.E5M2) * np.float64(h["do"][1])
    pt = fp8.decode(fp8.encode_sat(np.float32(448.0 / np.arange(1, S + 1)), fp8.E4M3), fp8.E4M3) / 448.0
    want = np.stack([(pt[j:, None] * do[j:]).sum(0) for j in range(S)])
    assert np.allclose(dV, want, rtol=1e-12, atol=1e-18)
    assert np.array_equal(dK, np.zeros_like(dK))             # dK = s dS^T Q with Q = 0

"""CPU checks of the test helper that bounds the FP8 matrix instruction's truncation (tests/mfma_model.py).

`dot_uncertainty` must bound what ANY plausible form of the device's accumulation can lose: the
measurements (tests/test_gpu_mfma_model.py) fix the group size and the number of kept places but not
the direction in which dropped bits go.  Here three exact integer models of a 13-place accumulation
(drop towards zero, drop towards minus infinity, round to nearest even), evaluated in rational
arithmetic on small random FP8 vectors, are each held against the bound.
"""
from fractions import Fraction
import math

import numpy as np
import pytest

from oracle import fp8
import mfma_model
from test_oracle_attention import make_head


def _quantise(x, quantum, mode):
    """Exact: x (Fraction) to a multiple of quantum (Fraction)."""
    n = x / quantum
    if mode == "zero":
        k = math.trunc(n)
    elif mode == "floor":
        k = math.floor(n)
    else:                                   # nearest, ties to even
        k = math.floor(n)
        r = n - k
        if r > Fraction(1, 2) or (r == Fraction(1, 2) and k % 2 == 1):
            k += 1
    return k * quantum


def device_like_dot(a, b, mode, keep=13, group=8):
    """Sum over groups of `group` indices of the products quantised to 2^(e_max - keep), e_max the exponent
    of the group's largest product; group sums added exactly.  a, b: lists of Fractions."""
    total = Fraction(0)
    for g0 in range(0, len(a), group):
        prods = [x * y for x, y in zip(a[g0:g0 + group], b[g0:g0 + group])]
        big = max(abs(p) for p in prods)
        if big == 0:
            continue
        e_max = math.floor(math.log2(big))
        while Fraction(2) ** e_max > big:
            e_max -= 1
        while Fraction(2) ** (e_max + 1) <= big:
            e_max += 1
        quantum = Fraction(2) ** (e_max - keep)
        total += sum(_quantise(p, quantum, mode) for p in prods)
    return total


def _random_codes(rng, n, fmt, spread):
    """Finite codes whose exponents spread over `spread` binades (wide spreads are what loses bits)."""
    emax_field = 15 if fmt == fp8.E4M3 else 30
    mb = 3 if fmt == fp8.E4M3 else 2
    e = rng.integers(max(0, emax_field - spread), emax_field + 1, size=n)
    m = rng.integers(0, 1 << mb, size=n)
    c = (e << mb) | m
    if fmt == fp8.E4M3:
        c = np.where(c == 0x7F, 0x7E, c)
    c = c | (rng.integers(0, 2, size=n) << 7)
    return c.astype(np.uint8)


@pytest.mark.parametrize("mode", ["zero", "floor", "nearest"])
@pytest.mark.parametrize("fmt_a", [fp8.E4M3, fp8.E5M2])
def test_bound_covers_every_13_place_accumulation_model(mode, fmt_a):
    rng = np.random.default_rng(13 + fmt_a)
    worst = 0.0
    for trial in range(150):
        D = int(rng.choice([8, 16, 32, 64]))
        spread = int(rng.integers(1, 16))
        ca, cb = _random_codes(rng, D, fmt_a, spread), _random_codes(rng, D, fp8.E4M3, spread)
        a, b = fp8.decode(ca, fmt_a), fp8.decode(cb, fp8.E4M3)
        fa, fb = [Fraction(float(v)) for v in a], [Fraction(float(v)) for v in b]
        exact = sum(x * y for x, y in zip(fa, fb))
        got = device_like_dot(fa, fb, mode)
        bound = mfma_model.dot_uncertainty(a[None, :], b[None, :])[0, 0]
        err = abs(got - exact)
        assert err <= Fraction(float(bound)), (trial, mode, float(err), bound)
        if bound > 0:
            worst = max(worst, float(err) / bound)
    assert 0.0 < worst <= 1.0                 # the models do lose bits on these inputs, and never more than the bound


def test_truncation_count_on_hand_built_groups_and_slack_properties():
    """The bound is zero when every product of a group sits within the kept window and counts one unit of
    the window's last place per product that can lose bits; the slack it induces is monotone in the window."""
    A = np.array([[1.0, 1.0, 0.5, 2.0, 1.0, 1.0, 1.0, 1.0] * 2])
    B = np.ones((1, 16))
    assert mfma_model.dot_uncertainty(A, B)[0, 0] == 0.0
    A2 = A.copy(); A2[0, 0] = 2.0 ** 12                      # group 0 now holds a product 2^12 times the others
    u = mfma_model.dot_uncertainty(A2, B)[0, 0]
    assert u == 7 * 2.0 ** (12 - mfma_model.MFMA_KEEP_BITS)   # seven small products, one unit each; group 1 untouched
    h = make_head(41, 64, 16)
    args = (h["q"][0], h["k"][0], h["v"][0], h["q"][1], h["k"][1], h["v"][1], 0.25, 448.0, True)
    slack = mfma_model.fwd_cast_slack(*args)
    assert slack.shape == (64, 16) and np.all(slack >= 0) and np.isfinite(slack).all()
    keep = mfma_model.MFMA_KEEP_BITS
    try:
        mfma_model.MFMA_KEEP_BITS = 6                        # a coarser window can only widen the set of two-code casts
        wide = mfma_model.fwd_cast_slack(*args)
    finally:
        mfma_model.MFMA_KEEP_BITS = keep
    assert np.all(wide >= slack) and wide.sum() > slack.sum()
    assert np.all(slack <= np.abs(fp8.decode(h["v"][0], fp8.E4M3)).max() * float(h["v"][1]))


def test_slack_is_what_flipping_the_two_code_elements_does():
    """Flip, by hand, every element of P that the model calls two-coded to its other code: the output moves
    by no more than the slack (the slack is the exact linear effect of those flips, summed in magnitude)."""
    from oracle import attention
    h = make_head(5, 48, 16)
    s, rho_p = 0.25, 448.0
    Q8, K8, V8, sq, sk, sv = h["q"][0], h["k"][0], h["v"][0], h["q"][1], h["k"][1], h["v"][1]
    O, _, _ = attention.attn_fwd_head(Q8, K8, V8, sq, sk, sv, s, rho_p, True)
    dx = mfma_model.logit_uncertainty(Q8, K8, sq, sk, s, True)
    slack = mfma_model.fwd_cast_slack(Q8, K8, V8, sq, sk, sv, s, rho_p, True, dx=dx)
    x = attention.logits(Q8, K8, sq, sk, s, True)
    M = np.ceil(x.max(axis=1, keepdims=True))
    for sign in (+1.0, -1.0):                                # push every logit to one end of its uncertainty
        p = np.exp2(x + sign * dx - M)
        l = np.exp2(x - M).sum(axis=1, keepdims=True)        # the row sum is held (its motion is the slack's second term)
        pq = fp8.decode(fp8.encode_sat((rho_p * p).astype(np.float32), fp8.E4M3), fp8.E4M3)
        O2 = np.float64(sv) * (pq @ fp8.decode(V8, fp8.E4M3)) / (rho_p * l)
        assert np.all(np.abs(O2 - O) <= slack + 1e-12)

"""Pins for abs-max, scale and cast (CPU only)."""
import numpy as np
import pytest
import torch

from oracle import bf16, fp8, scaling
from paper_2505_20524_amd import synth


def test_amax_invariants_and_planted_maximum():
    rng = np.random.default_rng(1)
    x = synth.f32_to_bf16_bits(rng.standard_normal(10007).astype(np.float32))
    a = scaling.amax(x)
    assert a == np.float32(np.abs(synth.bf16_bits_to_f32(x)).max())
    assert scaling.amax(x ^ np.uint16(0x8000)) == a                # sign flip
    assert scaling.amax(rng.permutation(x)) == a                   # permutation
    for pos in (0, 1, 4095, 10006):
        y = x.copy()
        y[pos] = 0xC2C8                                            # -100.0 in bf16
        assert scaling.amax(y) == np.float32(100.0)
    assert scaling.amax(np.zeros(5, np.uint16)) == 0
    assert scaling.amax(np.zeros(0, np.uint16)) == 0


@pytest.mark.parametrize("fmt", [fp8.E4M3, fp8.E5M2])
def test_scale_closed_form(fmt):
    # rho = FP8MaxValue / (2^m max H), Appendix E; powers of two make the quotient exact
    mx = fp8.fp8_max(fmt)
    for a, m in [(1.0, 0), (0.5, 0), (448.0, 0), (2.0 ** -20, 0), (3.0, 0), (1.0, 1), (7.0, 2)]:
        rho, rinv = scaling.compute_scale(np.float32(a), fmt, m)
        want = np.float32(np.float64(mx) / (np.float64(a) * 2 ** m))   # single rounding of the exact quotient
        assert rho == want and rho.dtype == np.float32
        assert rinv == np.float32(1.0 / np.float64(rho))
    assert scaling.compute_scale(np.float32(0), fmt)[0] == 1
    assert scaling.compute_scale(np.float32(np.inf), fmt)[0] == 1
    assert scaling.compute_scale(np.float32(np.nan), fmt)[0] == 1
    rho, rinv = scaling.compute_scale(np.float32(1e-44), fmt)
    assert np.isfinite(rho) and rho == np.finfo(np.float32).max
    # the abs-max element lands exactly on the largest finite code
    rng = np.random.default_rng(5)
    x = synth.f32_to_bf16_bits((rng.standard_normal(4096) * 3.7).astype(np.float32))
    rho, _ = scaling.compute_scale(scaling.amax(x), fmt)
    q = scaling.quantize(x, rho, fmt)
    assert (q & 0x7F).max() == (0x7E if fmt == fp8.E4M3 else 0x7B)


@pytest.mark.parametrize("fmt,tt", [(fp8.E4M3, torch.float8_e4m3fn), (fp8.E5M2, torch.float8_e5m2)])
def test_quantize_is_codec_of_binary32_product_and_transposes(fmt, tt):
    rng = np.random.default_rng(9)
    x = synth.f32_to_bf16_bits(rng.standard_normal((37, 53)).astype(np.float32) * 5)
    rho = np.float32(13.37)
    q, qT = scaling.quantize_with_transpose(x, rho, fmt)
    # library route: torch does the binary32 product and the cast
    xt = torch.from_numpy(synth.bf16_bits_to_f32(x).copy())
    mx = fp8.fp8_max(fmt)
    lib = (xt * torch.tensor(rho)).clamp(-mx, mx).to(tt).view(torch.uint8).numpy()
    assert np.array_equal(q, lib)
    assert np.array_equal(qT, lib.T) and qT.flags["C_CONTIGUOUS"] and qT.shape == (53, 37)
    # the product is rounded to binary32 BEFORE the FP8 rounding: build a case where that matters.
    # x*rho exactly representable only in float64, sitting a hair under an FP8 midpoint in float64
    # but rounding onto the midpoint (tie -> even) in binary32.
    xb = np.array([0x3F80], np.uint16)                              # 1.0
    mid = np.float32(1.0625)                                        # E4M3 midpoint between 1.0 and 1.125
    r = np.nextafter(np.float32(mid), np.float32(0))                # just below -> 1.0 (0x38)
    assert scaling.quantize(xb, r, fp8.E4M3)[0] == 0x38
    assert scaling.quantize(xb, mid, fp8.E4M3)[0] == 0x38           # tie -> even (0x38)
    xb3 = np.array([0x4040], np.uint16)                             # 3.0
    r3 = np.float32(1.1875 / 3.0)                                   # 3*r3 in binary32 vs exact
    t = np.float32(np.float32(3.0) * r3)
    assert scaling.quantize(xb3, r3, fp8.E4M3)[0] == fp8.encode_sat(t, fp8.E4M3)


def test_theorem_outliers_coarsen_the_rest():
    """Appendix C, Theorem 1: a larger outlier narrows the scaled range of the other entries, and the
    narrower range holds fewer representable FP8 numbers."""
    rng = np.random.default_rng(11)
    base = rng.standard_normal(4096).astype(np.float32)
    sigma = np.sqrt(np.mean(base ** 2))
    grid = np.abs(fp8.decode(np.arange(0x7F, dtype=np.uint8), fp8.E4M3))
    prev = None
    for tau in (4, 16, 64, 183, 688, 4000):
        x = base.copy()
        x[0] = tau * sigma
        xb = synth.f32_to_bf16_bits(x)
        rho, _ = scaling.compute_scale(scaling.amax(xb), fp8.E4M3)
        q = scaling.quantize(xb, rho, fp8.E4M3)[1:]
        span = np.abs(fp8.decode(q, fp8.E4M3)).max()           # scaled range of x_T
        bound = 448.0 * np.abs(synth.bf16_bits_to_f32(xb)[1:]).max() / (tau * sigma)
        assert span <= bound * 1.07                               # r m / (tau sigma), up to one rounding
        avail = int((grid <= span).sum())                         # representable magnitudes in that range
        used = len(np.unique(q & 0x7F))
        assert used <= avail
        if prev is not None:
            assert span < prev[0] and avail < prev[1]
        prev = (span, avail)
    assert prev[1] < 50                                            # of 127 magnitudes


def test_delayed_scaling_history():
    h = np.array([1.0, 5.0, 2.0, 0.5], np.float32)
    rho, _ = scaling.history_scale(h, fp8.E4M3)
    assert rho == np.float32(448.0 / 5.0)
    h2 = scaling.history_update(h, 0.25)
    assert np.array_equal(h2, np.array([0.25, 1.0, 5.0, 2.0], np.float32))
    for _ in range(2):
        h2 = scaling.history_update(h2, 0.25)
    assert scaling.history_scale(h2, fp8.E4M3)[0] == np.float32(448.0)   # the 5.0 has left the window... 

"""Pins of the QK-RMSNorm + cast oracle (Section 3 of the paper; cast of Appendix E)."""
import numpy as np
import torch

from oracle import bf16, fp8, qknorm, scaling
from paper_2505_20524_amd import synth


def bits(x):
    return synth.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def test_closed_forms():
    D = 128
    # constant vector: every element has magnitude rms, so y = gain * sign
    y = qknorm.normalize(bits(np.full((3, D), -2.5)), gain=1.5)
    assert np.array_equal(y, np.full((3, D), -1.5))
    # one-hot vector: rms = |a| / sqrt(D), so the hot element becomes sqrt(D) whatever its size
    x = np.zeros((2, D), np.float32); x[0, 5] = 3.0; x[1, 77] = -0.125
    y = qknorm.normalize(bits(x))
    assert np.isclose(y[0, 5], np.sqrt(D), rtol=1e-15) and np.isclose(y[1, 77], -np.sqrt(D), rtol=1e-15) and np.count_nonzero(y) == 2
    # +-a pattern with k non-zeros: |y| = sqrt(D / k)
    x = np.zeros((1, D), np.float32); x[0, :32] = 7.0; x[0, 32:64] = -7.0
    assert np.allclose(np.abs(qknorm.normalize(bits(x))[0, :64]), np.sqrt(D / 64), rtol=0, atol=1e-15)
    # zero vector -> zeros (no epsilon in the paper's formula), abs-max of an all-zero tensor is 0
    assert not qknorm.normalize(bits(np.zeros((2, D)))).any()
    assert qknorm.amax(bits(np.zeros((2, D)))) == 0.0


def test_unit_rms_scale_invariance_and_bound():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((64, 128)).astype(np.float32)
    x[:, 3] *= 40.0
    xb = bits(x)
    y = qknorm.normalize(xb, gain=0.75)
    assert np.allclose(np.sqrt(np.mean(y * y, axis=1)), 0.75, rtol=1e-12)        # rms(y) = gain
    # invariant to a power-of-two rescaling of a row (exact in bf16), odd in x
    assert np.array_equal(qknorm.normalize(bits(x * 4.0), 0.75), y)
    assert np.array_equal(qknorm.normalize(bits(-x), 0.75), -y)
    # |y_i| <= gain sqrt(D), with equality only for one-hot rows: the static bound behind a fixed scale
    assert qknorm.amax(xb, 0.75) <= 0.75 * np.sqrt(128)
    # against torch: x / sqrt(mean(x^2)) in float64
    t = torch.from_numpy(bf16.bits_to_f64(xb))
    ref = (0.75 * t / t.pow(2).mean(dim=1, keepdim=True).sqrt()).numpy()
    assert np.allclose(y, ref, rtol=1e-14, atol=0)


def test_quantize_is_the_cast_of_the_normalised_tensor():
    """The codes are those of the ordinary per-tensor cast (pinned on its own) applied to y, when y
    happens to be bf16-exact; and the window brackets the point cast."""
    D = 128
    x = np.zeros((4, D), np.float32)
    x[0, :] = 3.0; x[1, ::2] = 1.0; x[1, 1::2] = -1.0; x[2, 9] = 5.0; x[3, :64] = 0.5    # y in {+-1, sqrt(D) (not exact), sqrt(2)}
    xb = bits(x)
    for fmt in (fp8.E4M3, fp8.E5M2):
        rho = np.float32(fp8.fp8_max(fmt) / 16.0)
        q = qknorm.quantize(xb, rho, fmt)
        yb = bits(qknorm.normalize(xb)[:2])                       # rows 0, 1: y = +-1 exactly
        assert np.array_equal(q[:2], scaling.quantize(yb, rho, fmt))
        lo, hi = qknorm.quantize_window(xb, rho, fmt)
        d = lambda c: fp8.decode(c, fmt)
        assert np.all(np.abs(d(lo)) <= np.abs(d(q))) and np.all(np.abs(d(q)) <= np.abs(d(hi)))
        # saturation: the one-hot row maps to sqrt(D) * rho > max -> the largest code, with its sign
        big = qknorm.quantize(xb, np.float32(fp8.fp8_max(fmt)), fmt)
        assert d(big)[2, 9] == fp8.fp8_max(fmt)
    # the window is narrow: on random data only a handful of elements are undecided
    rng = np.random.default_rng(1)
    xb = bits(rng.standard_normal((256, D)))
    lo, hi = qknorm.quantize_window(xb, np.float32(30.0), fp8.E4M3)
    assert 0 <= np.count_nonzero(lo != hi) <= 20

"""Pins of the post-RMSNorm + residual oracle (Section 3: post-normalised block with a trainable gains vector)."""
import numpy as np
import torch

from oracle import bf16, postnorm
from paper_2505_20524_amd import synth


def _bits(a):
    return synth.f32_to_bf16_bits(np.asarray(a, np.float32))


def test_closed_forms():
    D = 8
    g = np.arange(1, D + 1, dtype=np.float32) / 4
    # constant vector c: rms = |c|, N = sign(c) gamma
    n = postnorm.normalize(_bits(np.full((1, D), -3.0)), g)
    assert np.array_equal(n, -g[None, :].astype(np.float64))
    # one-hot at position k: rms = |v| / sqrt(D), N = gamma_k sqrt(D) at k and 0 elsewhere
    x = np.zeros((1, D), np.float32)
    x[0, 5] = 0.5
    n = postnorm.normalize(_bits(x), g)
    assert np.isclose(n[0, 5], g[5] * np.sqrt(D), rtol=1e-15) and np.count_nonzero(n) == 1
    # zero vector adds nothing (no epsilon in the formula)
    xres = _bits(np.linspace(-1, 1, D)[None, :])
    assert np.array_equal(postnorm.residual_bf16(xres, _bits(np.zeros((1, D))), g), xres)
    # gains of one: the normalised vector has unit rms; positive rescaling of y changes nothing
    rng = np.random.default_rng(0)
    y = rng.standard_normal((5, 64)).astype(np.float32)
    n = postnorm.normalize(_bits(y), np.ones(64, np.float32))
    assert np.allclose(np.sqrt(np.mean(n * n, axis=-1)), 1.0, rtol=1e-14)
    assert np.array_equal(postnorm.normalize(_bits(y), g64 := rng.random(64).astype(np.float32)),
                          postnorm.normalize(_bits(bf16.bits_to_f64(_bits(y)) * 4.0), g64))
    # the gain multiplies channel-wise (a transposed or row-wise broadcast would fail this)
    e = np.zeros(64, np.float32)
    e[7] = 1.0
    only7 = postnorm.normalize(_bits(y), e)
    assert np.count_nonzero(only7[:, :7]) == 0 and np.count_nonzero(only7[:, 8:]) == 0 and np.all(only7[:, 7] != 0)


def test_against_torch_and_sign_of_the_residual():
    rng = np.random.default_rng(1)
    rows, D = 7, 96
    xb, yb = _bits(rng.standard_normal((rows, D))), _bits(rng.standard_normal((rows, D)) * 3)
    g = (rng.random(D).astype(np.float32) + 0.5) / 4
    xt = torch.from_numpy(bf16.bits_to_f64(xb))
    yt = torch.from_numpy(bf16.bits_to_f64(yb))
    ref = xt + torch.from_numpy(g.astype(np.float64)) * yt * torch.rsqrt(yt.pow(2).mean(-1, keepdim=True))
    got = postnorm.residual(xb, yb, g)
    assert np.allclose(got, ref.numpy(), rtol=1e-14, atol=1e-15)
    # it is a sum, not a difference, and x enters unscaled
    assert np.allclose(got - bf16.bits_to_f64(xb), postnorm.normalize(yb, g), rtol=0, atol=1e-15)
    # torch.nn.functional.rms_norm (eps tiny) as a second route to N_gamma
    n2 = torch.nn.functional.rms_norm(yt, (D,), weight=torch.from_numpy(g.astype(np.float64)), eps=1e-300).numpy()
    assert np.allclose(postnorm.normalize(yb, g), n2, rtol=1e-13, atol=0)


def test_window_brackets_the_rounded_sum():
    rng = np.random.default_rng(2)
    xb, yb = _bits(rng.standard_normal((32, 128))), _bits(rng.standard_normal((32, 128)))
    g = np.full(128, 0.25, np.float32)
    mid = postnorm.residual_bf16(xb, yb, g)
    lo, hi = postnorm.residual_window(xb, yb, g)
    v, vl, vh = (bf16.bits_to_f64(b) for b in (mid, lo, hi))
    assert np.all(vl <= v) and np.all(v <= vh)
    assert np.mean(lo != hi) < 2e-3                      # a 2^-20 window rarely straddles a bf16 rounding boundary
    # the ends are at most one bf16 step apart
    assert np.all(np.abs(vh - vl) <= np.abs(v) * 2.0 ** -7 + 1e-40)

"""Pins of the GeLU + cast and tanh_alpha + cast oracles (Section 3, architecture suite; cast of Appendix E)."""
import math

import numpy as np
import torch
from scipy import integrate

from oracle import fp8, gelu, scaling
from paper_2505_20524_amd import synth


def test_gelu_is_x_times_the_normal_distribution_function():
    # Phi by numerical integration of the density, independent of erf / erfc
    for x in (-3.0, -1.0, -0.25, 0.5, 2.0):
        phi, _ = integrate.quad(lambda t: math.exp(-0.5 * t * t) / math.sqrt(2 * math.pi), -np.inf, x, epsabs=1e-14, epsrel=1e-13)
        assert np.isclose(gelu.gelu(x), x * phi, rtol=1e-10, atol=0)
    # printed constants of the normal distribution: Phi(1) = 0.8413447460685429
    assert np.isclose(gelu.gelu(1.0), 0.8413447460685429, rtol=1e-15)
    assert np.isclose(gelu.gelu(-1.0), -0.15865525393145707, rtol=1e-14)
    assert gelu.gelu(0.0) == 0.0


def test_gelu_identities():
    x = np.linspace(-9, 9, 3601)
    y = gelu.gelu(x)
    # Phi(x) + Phi(-x) = 1  =>  GeLU(x) - GeLU(-x) = x
    assert np.allclose(y - gelu.gelu(-x), x, rtol=4e-16, atol=1e-16)
    # bounds: x Phi(x) lies between min(x, 0) and max(x, 0); one minimum of about -0.17 near x = -0.75
    assert np.all(y <= np.maximum(x, 0) + 1e-16) and np.all(y >= np.minimum(x, 0))
    k = int(np.argmin(y))
    assert abs(x[k] + 0.7518) < 0.005 and abs(y[k] + 0.169971) < 1e-5
    # far tails: identity on the right; on the left the Mills-ratio asymptote x Phi(x) ~ -phi(x) (1 - 1/x^2)
    assert np.isclose(gelu.gelu(12.0), 12.0, rtol=1e-15)
    xl = -12.0
    dens = math.exp(-0.5 * xl * xl) / math.sqrt(2 * math.pi)
    assert np.isclose(gelu.gelu(xl), -dens * (1 - 1 / xl ** 2 + 3 / xl ** 4), rtol=1e-3)
    # derivative Phi(x) + x phi(x)
    d = np.gradient(y, x)
    dens = np.exp(-0.5 * x * x) / np.sqrt(2 * np.pi)
    assert np.allclose(d[1:-1], (y / np.where(x == 0, 1, x) + x * dens)[1:-1] + (x[1:-1] == 0) * 0.5, atol=2e-5)
    # torch's exact form in float64 (written with 1 + erf, so its far-negative tail cancels to 0: absolute bound)
    ref = torch.nn.functional.gelu(torch.from_numpy(x), approximate="none").numpy()
    assert np.allclose(y, ref, rtol=1e-14, atol=1e-15)


def test_tanh_alpha():
    a = 0.7
    x = np.linspace(-30, 30, 2401)
    y = gelu.tanh_alpha(x, a)
    # definition through the exponential, written without tanh
    e = np.expm1(2 * a * x)
    with np.errstate(invalid="ignore", over="ignore"):
        ref = np.where(np.isfinite(e), e / (e + 2.0), 1.0)
    assert np.allclose(y, ref, rtol=1e-14, atol=1e-16)
    assert np.array_equal(y, -gelu.tanh_alpha(-x, a))                      # odd
    assert np.all(np.abs(y) <= 1.0) and np.all(np.diff(y) >= 0)            # bounded, monotone
    assert np.allclose(np.arctanh(y[np.abs(a * x) < 5]), a * x[np.abs(a * x) < 5], rtol=1e-9, atol=1e-12)
    assert np.isclose(gelu.tanh_alpha(1e-6, a), a * 1e-6, rtol=1e-11)      # slope alpha at the origin
    assert np.isclose(gelu.tanh_alpha(1.0, 1.0), 0.7615941559557649, rtol=1e-15)
    assert np.allclose(y, torch.tanh(a * torch.from_numpy(x)).numpy(), rtol=1e-14, atol=0)
    # alpha = 0 maps everything to 0
    assert not gelu.tanh_alpha(x, 0.0).any()


def test_casts_are_the_per_tensor_cast_of_the_activated_values():
    # tanh: inputs whose image is bf16-exact do not exist apart from 0 and the saturated ends, so use those
    xb = synth.f32_to_bf16_bits(np.array([[0.0, 60.0, -60.0, -0.0]], np.float32))
    for fmt in (fp8.E4M3, fp8.E5M2):
        q = gelu.tanh_quantize(xb, np.float32(448.0), fmt, 1.0)
        ref = scaling.quantize(synth.f32_to_bf16_bits(np.array([[0.0, 1.0, -1.0, -0.0]], np.float32)), np.float32(448.0), fmt)
        assert np.array_equal(q, ref)
        lo, hi = gelu.tanh_window(xb, np.float32(448.0), fmt, 1.0)
        assert np.array_equal(lo, q) and np.array_equal(hi, q)
    assert gelu.tanh_amax(xb, 1.0) == 1.0
    # GeLU: far right it is the identity (Phi rounds to 1 in float64 beyond x ~ 8.3), far left exactly 0 after the cast
    x = np.array([[0.0, 10.0, 16.0, 40.0, -40.0, -16.0]], np.float32)
    xb = synth.f32_to_bf16_bits(x)
    for fmt in (fp8.E4M3, fp8.E5M2):
        rho = np.float32(8.0)
        q = gelu.gelu_quantize(xb, rho, fmt)
        ref = scaling.quantize(synth.f32_to_bf16_bits(np.array([[0.0, 10.0, 16.0, 40.0, -0.0, -0.0]], np.float32)), rho, fmt)
        assert np.array_equal(q, ref)
        lo, hi = gelu.gelu_window(xb, rho, fmt)
        assert np.array_equal(lo, q) and np.array_equal(hi, q)
    assert gelu.gelu_amax(xb) == 40.0


def test_windows_bracket_the_point_cast_and_are_rarely_open():
    rng = np.random.default_rng(5)
    xb = synth.f32_to_bf16_bits(rng.standard_normal((64, 256)).astype(np.float32) * 2)
    for fmt in (fp8.E4M3, fp8.E5M2):
        for q, (lo, hi) in ((gelu.gelu_quantize(xb, np.float32(30.0), fmt), gelu.gelu_window(xb, np.float32(30.0), fmt)),
                            (gelu.tanh_quantize(xb, np.float32(448.0), fmt, 0.5), gelu.tanh_window(xb, np.float32(448.0), fmt, 0.5))):
            v, vl, vh = (fp8.decode(c, fmt) for c in (q, lo, hi))
            assert np.all(np.minimum(vl, vh) <= v) and np.all(v <= np.maximum(vl, vh))
            # open windows are rare; most are exact ties of small bf16 inputs in tanh's linear regime
            assert np.mean(lo != hi) < 5e-3

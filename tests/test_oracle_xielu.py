"""Pins of the xIELU + cast oracle (Appendix B, equation xIELU; cast of Appendix E)."""
import numpy as np
import torch

from oracle import fp8, scaling, xielu
from paper_2505_20524_amd import synth


def test_values_and_branches():
    ap, an = 0.8, 0.6
    # hand-evaluated points of the equation
    assert xielu.xielu(2.0, ap, an) == ap * 4.0 + 1.0
    assert xielu.xielu(0.0, ap, an) == 0.0
    assert np.isclose(xielu.xielu(-1.0, ap, an), an * (np.exp(-1.0) - 1.0) + an - 0.5, rtol=1e-15)
    # continuous and once differentiable at 0 (slope 0.5 on both sides), as an ELU-type extension must be
    h = 1e-6
    assert abs(xielu.xielu(h, ap, an) - xielu.xielu(-h, ap, an) - h) < 1e-11
    # alpha_p = alpha_n = 0 leaves 0.5 x; alpha_n = 0 is a squared-ReLU plus a linear term
    x = np.linspace(-4, 4, 101)
    assert np.array_equal(xielu.xielu(x, 0.0, 0.0), 0.5 * x)
    assert np.allclose(xielu.xielu(x, ap, 0.0), ap * np.maximum(x, 0) ** 2 + 0.5 * x, rtol=1e-15, atol=0)
    # far negative: e^x vanishes, the function runs along (0.5 - alpha_n) x - alpha_n
    assert np.isclose(xielu.xielu(-50.0, ap, an), (0.5 - an) * -50.0 - an, rtol=1e-15)
    # small negative x: alpha_n (e^x - 1 - x) = alpha_n x^2 / 2 + O(x^3), no cancellation in the oracle
    xs = -1e-5
    assert np.isclose(xielu.xielu(xs, ap, an) - 0.5 * xs, an * xs * xs / 2, rtol=1e-4)


def test_against_torch_autograd_free_formula_and_monotone_regions():
    ap, an = 0.8, 0.8
    x = torch.linspace(-6, 6, 2001, dtype=torch.float64)
    ref = torch.where(x > 0, ap * x * x + 0.5 * x, an * torch.expm1(x) - an * x + 0.5 * x).numpy()
    assert np.allclose(xielu.xielu(x.numpy(), ap, an), ref, rtol=1e-14, atol=1e-16)
    # derivative: 2 alpha_p x + 0.5 for x > 0 (increasing), alpha_n (e^x - 1) + 0.5 for x <= 0
    y = xielu.xielu(x.numpy(), ap, an)
    d = np.gradient(y, x.numpy())
    xn = x.numpy()
    assert np.allclose(d[1001:-1], 2 * ap * xn[1001:-1] + 0.5, atol=1e-4)
    assert np.allclose(d[1:999], an * np.expm1(xn[1:999]) + 0.5, atol=1e-4)


def test_quantize_is_the_cast_of_the_activated_tensor():
    """On inputs whose activation is bf16-exact the codes are those of the per-tensor cast (pinned on its own)."""
    ap, an = 0.5, 0.0
    x = np.array([[0.0, 1.0, 2.0, 4.0, -1.0, -2.0, -8.0, 0.5]], np.float32)     # y = 0, 1, 3, 10, -.5, -1, -4, .375
    xb = synth.f32_to_bf16_bits(x)
    y = xielu.activate(xb, ap, an)
    assert np.array_equal(y, np.array([[0.0, 1.0, 3.0, 10.0, -0.5, -1.0, -4.0, 0.375]]))
    for fmt in (fp8.E4M3, fp8.E5M2):
        rho = np.float32(16.0)
        q = xielu.quantize(xb, rho, fmt, ap, an)
        assert np.array_equal(q, scaling.quantize(synth.f32_to_bf16_bits(y.astype(np.float32)), rho, fmt))
        lo, hi = xielu.quantize_window(xb, rho, fmt, ap, an)
        assert np.array_equal(lo, q) and np.array_equal(hi, q)          # exact values sit in the middle of their cells
    assert xielu.amax(xb, ap, an) == 10.0
    # saturation keeps the sign
    big = xielu.quantize(synth.f32_to_bf16_bits(np.array([[100.0, -3000.0]], np.float32)), np.float32(1.0), fp8.E4M3, 1.0, 0.0)
    assert fp8.decode(big, fp8.E4M3).tolist() == [[448.0, -448.0]]

"""GPU parity: GeLU and tanh_alpha fused with the FP8 cast against the float64 oracle.

The activated tensor is never stored, so a code is a rounding decision on a binary32 value; the
oracle gives, per element, the codes at both ends of a relative window (2^-19, for GeLU widened by
x^2 2^-23 on the negative side).  Where they coincide the GPU byte must equal them; elsewhere it
must be one of the two.
"""
import numpy as np
import pytest
import torch

from oracle import fp8, gelu
from paper_2505_20524_amd import fog, synth
from parity import dev, fscalar

pytestmark = pytest.mark.gpu

SHAPES = [(1, 16, 0), (64, 256, 0), (333, 1024, 0), (100, 272, 16), (7, 17, 3), (50, 100, 0), (1024, 8192, 0),
          (4100, 7168, 0), (8200, 2064, 16)]       # the last two: several trips per workgroup at the largest grid


def run(kind, xb, cols, fmt, rho, alpha, pad_q):
    rows = xb.shape[0]
    x = dev(xb)
    if xb.shape[1] != cols:
        x = x[:, :cols]
    qfull = torch.full((rows, cols + pad_q), 0xAA, dtype=torch.uint8, device="cuda")
    q = qfull[:, :cols] if pad_q else qfull
    am = torch.full((1,), -1.0, device="cuda")
    if kind == "gelu":
        fog.gelu_quantize(x, fmt, fscalar(rho), q, amax_out=am)
    else:
        fog.tanh_quantize(x, alpha, fmt, fscalar(rho), q, amax_out=am)
    torch.cuda.synchronize()
    if pad_q:
        assert (qfull[:, cols:] == 0xAA).all()
    return q.cpu().numpy(), am.item()


def check(kind, xb, cols, fmt, rho, alpha=1.0, pad_q=0, max_open=5e-3):
    got, am = run(kind, xb, cols, fmt, rho, alpha, pad_q)
    view = xb[:, :cols]
    if kind == "gelu":
        lo, hi = gelu.gelu_window(view, rho, fmt)
        want = gelu.gelu_amax(view)
    else:
        lo, hi = gelu.tanh_window(view, rho, fmt, alpha)
        want = gelu.tanh_amax(view, alpha)
    undecided = lo != hi
    assert np.array_equal(got[~undecided], lo[~undecided])
    assert np.all((got[undecided] == lo[undecided]) | (got[undecided] == hi[undecided]))
    assert undecided.mean() <= max_open
    assert abs(am - want) <= 2.0 ** -19 * want
    return got


@pytest.mark.parametrize("fmt", [fp8.E4M3, fp8.E5M2])
@pytest.mark.parametrize("rows,cols,pad", SHAPES)
def test_gelu_parity(rows, cols, pad, fmt):
    rng = np.random.default_rng(rows + cols + fmt)
    x = (rng.standard_normal((rows, cols + pad)) * 2.0).astype(np.float32)
    x[:, 1 % cols] *= 8.0                                   # an outlier channel
    x[0, 0] = 0.0
    xb = synth.f32_to_bf16_bits(x)
    rho = np.float32(fp8.fp8_max(fmt) / max(gelu.gelu_amax(xb[:, :cols]), 1e-30))
    check("gelu", xb, cols, fmt, rho, pad_q=pad)


@pytest.mark.parametrize("fmt", [fp8.E4M3, fp8.E5M2])
@pytest.mark.parametrize("rows,cols,pad", SHAPES)
def test_tanh_parity(rows, cols, pad, fmt):
    rng = np.random.default_rng(rows + cols + fmt + 1)
    x = (rng.standard_normal((rows, cols + pad)) * 2.0).astype(np.float32)
    x[:, 1 % cols] *= 8.0
    x[0, 0] = 0.0
    xb = synth.f32_to_bf16_bits(x)
    alpha = 0.5 if rows % 2 else -1.25                      # the trainable scalar may change sign
    check("tanh", xb, cols, fmt, np.float32(fp8.fp8_max(fmt)), alpha=alpha, pad_q=pad)      # |y| <= 1: the constant scale


def test_tails_small_magnitudes_and_errors():
    # GeLU's negative tail down to x = -12 under a huge scale (values of 1e-30 land on real codes only then), tiny |x|
    x = np.concatenate([-np.linspace(0.0, 12.0, 512, dtype=np.float32), np.logspace(-6, 1, 512, dtype=np.float32)]).reshape(8, 128)
    xb = synth.f32_to_bf16_bits(np.concatenate([x, -x]))
    check("gelu", xb, 128, fp8.E5M2, np.float32(2.0 ** 60), max_open=2e-2)
    got = check("gelu", xb, 128, fp8.E4M3, np.float32(1e4), max_open=2e-2)
    assert np.isfinite(fp8.decode(got, fp8.E4M3)).all()
    # tanh: tiny arguments (linear regime) and saturated ends
    check("tanh", xb, 128, fp8.E5M2, np.float32(2.0 ** 20), alpha=1.0, max_open=2e-2)
    got = check("tanh", xb, 128, fp8.E4M3, np.float32(448.0), alpha=30.0, max_open=2e-2)
    assert np.abs(fp8.decode(got, fp8.E4M3)).max() == 448.0
    check("tanh", xb, 128, fp8.E4M3, np.float32(448.0), alpha=0.0)
    lib = fog.load()
    st = torch.cuda.current_stream().cuda_stream
    xd = torch.zeros((4, 64), dtype=torch.int16, device="cuda")
    q = torch.zeros((4, 64), dtype=torch.uint8, device="cuda")
    f = fscalar(1.0)
    g, t = lib.fog_gelu_quantize, lib.fog_tanh_quantize
    assert g(xd.data_ptr(), 4, 64, 64, 0, None, q.data_ptr(), 64, None, st) == 1
    assert g(xd.data_ptr(), 4, 64, 64, 0, f.data_ptr(), None, 64, None, st) == 1
    assert g(xd.data_ptr(), 4, 64, 32, 0, f.data_ptr(), q.data_ptr(), 64, None, st) == 2
    assert g(xd.data_ptr() + 1, 4, 32, 32, 0, f.data_ptr(), q.data_ptr(), 32, None, st) == 3
    assert g(xd.data_ptr(), 4, 64, 64, 2, f.data_ptr(), q.data_ptr(), 64, None, st) == 4
    assert t(xd.data_ptr(), 4, 64, 64, float("inf"), 0, f.data_ptr(), q.data_ptr(), 64, None, st) == 4
    assert t(xd.data_ptr(), 4, 64, 64, float("nan"), 0, f.data_ptr(), q.data_ptr(), 64, None, st) == 4
    assert t(xd.data_ptr(), 4, 64, 64, 1.0, 0, None, q.data_ptr(), 64, None, st) == 1
    assert t(None, 0, 64, 64, 1.0, 0, f.data_ptr(), None, 64, f.data_ptr(), st) == 0
    torch.cuda.synchronize()
    assert f.item() == 0.0


@pytest.mark.parametrize("kind", ["gelu", "tanh"])
def test_nan_inputs_reach_the_codes_and_the_abs_max(kind):
    """A NaN activation input gives the NaN code (not the largest finite code the clamp alone would produce;
    the sign of a NaN that went through arithmetic is not defined) and a NaN abs-max, so a diverged tensor
    stays visible to the scaling history."""
    rng = np.random.default_rng(3)
    for rows, cols in ((64, 256), (7, 17)):                      # the vector path and the element-wise path
        xb = synth.f32_to_bf16_bits(rng.standard_normal((rows, cols)).astype(np.float32))
        xb[0, 0] = 0x7FC0
        xb[rows - 1, cols - 1] = 0xFFC0
        xb[rows // 2, 5] = 0x7FA1
        for fmt in (fp8.E4M3, fp8.E5M2):
            got, am = run(kind, xb, cols, fmt, 100.0, 0.7, 0)
            nan_codes = (got & 0x7F) == 0x7F
            assert nan_codes[0, 0] and nan_codes[rows - 1, cols - 1] and nan_codes[rows // 2, 5]
            assert nan_codes.sum() == 3
            assert np.isnan(am)

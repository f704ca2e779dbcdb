"""GPU parity: xIELU fused with the FP8 cast against the float64 oracle.

The activated tensor is never stored, so a code is a rounding decision on a binary32 value; the
oracle gives, per element, the codes at both ends of a 2^-19 relative window.  Where they coincide
the GPU byte must equal them; elsewhere (a few elements in 10^5) it must be one of the two.
"""
import numpy as np
import pytest
import torch

from oracle import fp8, xielu
from paper_2505_20524_amd import fog, synth
from parity import dev, fscalar

pytestmark = pytest.mark.gpu


def check(xb, cols, fmt, rho, ap, an, pad_q=0):
    rows = xb.shape[0]
    x = dev(xb)
    if xb.shape[1] != cols:
        x = x[:, :cols]
    qfull = torch.full((rows, cols + pad_q), 0xAA, dtype=torch.uint8, device="cuda")
    q = qfull[:, :cols] if pad_q else qfull
    am = torch.full((1,), -1.0, device="cuda")
    fog.xielu_quantize(x, ap, an, fmt, fscalar(rho), q, amax_out=am)
    torch.cuda.synchronize()
    if pad_q:
        assert (qfull[:, cols:] == 0xAA).all()
    got = q.cpu().numpy()
    view = xb[:, :cols]
    lo, hi = xielu.quantize_window(view, rho, fmt, ap, an)
    undecided = lo != hi
    assert np.array_equal(got[~undecided], lo[~undecided])
    assert np.all((got[undecided] == lo[undecided]) | (got[undecided] == hi[undecided]))
    assert undecided.mean() <= 1e-3
    want = xielu.amax(view, ap, an)
    assert abs(am.item() - want) <= 2.0 ** -19 * want
    return got


@pytest.mark.parametrize("fmt", [fp8.E4M3, fp8.E5M2])
@pytest.mark.parametrize("rows,cols,pad", [(1, 16, 0), (64, 256, 0), (333, 1024, 0), (100, 272, 16), (7, 17, 3), (50, 100, 0),
                                           (1024, 8192, 0), (4100, 7168, 0), (8200, 2064, 16)])
def test_xielu_parity(rows, cols, pad, fmt):
    rng = np.random.default_rng(rows + cols + fmt)
    x = (rng.standard_normal((rows, cols + pad)) * 2.0).astype(np.float32)
    x[:, 1 % cols] *= 8.0                                   # an outlier channel
    x[0, 0] = 0.0
    xb = synth.f32_to_bf16_bits(x)
    ap, an = (0.8, 0.8) if rows % 2 else (0.3, 1.5)
    rho = np.float32(fp8.fp8_max(fmt) / max(xielu.amax(xb[:, :cols], ap, an), 1e-30))
    check(xb, cols, fmt, rho, ap, an, pad_q=pad)


def test_xielu_small_magnitudes_saturation_and_errors():
    # |x| down to 1e-6: the quadratic term of the negative branch must not be lost to cancellation
    x = -np.logspace(-6, 1, 512, dtype=np.float32).reshape(4, 128)
    xb = synth.f32_to_bf16_bits(np.concatenate([x, -x]))
    check(xb, 128, fp8.E5M2, np.float32(2.0 ** 20), 0.8, 0.8)            # a huge scale: small values land on real codes, large ones saturate
    got = check(xb, 128, fp8.E4M3, np.float32(1e4), 0.8, 0.8)
    assert np.isfinite(fp8.decode(got, fp8.E4M3)).all()
    lib = fog.load()
    st = torch.cuda.current_stream().cuda_stream
    xd = torch.zeros((4, 64), dtype=torch.int16, device="cuda")
    q = torch.zeros((4, 64), dtype=torch.uint8, device="cuda")
    f = fscalar(1.0)
    call = lib.fog_xielu_quantize
    assert call(xd.data_ptr(), 4, 64, 64, 0.8, 0.8, 0, None, q.data_ptr(), 64, None, st) == 1
    assert call(xd.data_ptr(), 4, 64, 64, 0.8, 0.8, 0, f.data_ptr(), None, 64, None, st) == 1
    assert call(xd.data_ptr(), 4, 64, 32, 0.8, 0.8, 0, f.data_ptr(), q.data_ptr(), 64, None, st) == 2
    assert call(xd.data_ptr() + 1, 4, 32, 32, 0.8, 0.8, 0, f.data_ptr(), q.data_ptr(), 32, None, st) == 3
    assert call(xd.data_ptr(), 4, 64, 64, -0.1, 0.8, 0, f.data_ptr(), q.data_ptr(), 64, None, st) == 4
    assert call(xd.data_ptr(), 4, 64, 64, 0.8, 0.8, 2, f.data_ptr(), q.data_ptr(), 64, None, st) == 4
    assert call(None, 0, 64, 64, 0.8, 0.8, 0, f.data_ptr(), None, 64, f.data_ptr(), st) == 0
    torch.cuda.synchronize()
    assert f.item() == 0.0

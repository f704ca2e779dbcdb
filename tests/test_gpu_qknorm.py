"""GPU parity: QK RMS normalisation fused with the FP8 cast against the float64 oracle.

The normalised tensor is never stored, so a code is a rounding decision on a binary32 value; the
oracle gives, per element, the codes at both ends of a 2^-20 relative window.  Where they coincide
(all but a few elements in 10^5) the GPU byte must equal them; elsewhere it must be one of the two.
"""
import numpy as np
import pytest
import torch

from oracle import fp8, qknorm
from paper_2505_20524_amd import fog, synth
from parity import dev, fscalar

pytestmark = pytest.mark.gpu


def run(xb, cols, fmt, rho, gain, pad_q=0):
    rows = xb.shape[0]
    x = dev(xb)
    if xb.shape[1] != cols:
        x = x[:, :cols]
    qfull = torch.full((rows, cols + pad_q), 0xAA, dtype=torch.uint8, device="cuda")
    q = qfull[:, :cols] if pad_q else qfull
    am = torch.full((1,), -1.0, device="cuda")
    fog.rmsnorm_quantize(x, fmt, fscalar(rho), q, gain=gain, amax_out=am)
    torch.cuda.synchronize()
    if pad_q:
        assert (qfull[:, cols:] == 0xAA).all()              # nothing written past the row
    return q.cpu().numpy(), am.item()


def check(xb, cols, fmt, rho, gain, pad_q=0):
    q, am = run(xb, cols, fmt, rho, gain, pad_q)
    view = xb[:, :cols]
    lo, hi = qknorm.quantize_window(view, rho, fmt, gain)
    undecided = lo != hi
    assert np.array_equal(q[~undecided], lo[~undecided])
    assert np.all((q[undecided] == lo[undecided]) | (q[undecided] == hi[undecided]))
    assert undecided.mean() <= 1e-3
    want = qknorm.amax(view, gain)
    assert abs(am - want) <= 2.0 ** -20 * want
    return q


@pytest.mark.parametrize("fmt", [fp8.E4M3, fp8.E5M2])
@pytest.mark.parametrize("rows,cols,pad", [(1, 128, 0), (4, 128, 0), (1000, 128, 0), (8192, 128, 0), (333, 64, 0), (100, 256, 8),
                                           (65, 512, 0), (50, 100, 0), (7, 17, 3), (129, 136, 0)])
def test_qknorm_parity(rows, cols, pad, fmt):
    rng = np.random.default_rng(rows + cols + fmt)
    x = rng.standard_normal((rows, cols + pad)).astype(np.float32) * 10.0 ** rng.uniform(-2, 2, (rows, 1))
    x[:, 1 % cols] *= 30.0                               # an outlier channel: the case the normalisation is there for
    xb = synth.f32_to_bf16_bits(x)
    gain = 1.0 if rows % 2 else 0.8
    rho = np.float32(fp8.fp8_max(fmt) / (gain * np.sqrt(cols)))      # the scale that cannot saturate
    check(xb, cols, fmt, rho, gain, pad_q=pad)


def test_qknorm_special_rows_and_saturation():
    D = 128
    x = np.zeros((6, D), np.float32)
    x[1, :] = 2.0                                         # constant: y = 1
    x[2, 40] = -3.0                                       # one-hot: y = -sqrt(D)
    x[3, ::2] = 1.0; x[3, 1::2] = -1.0
    x[4, :] = np.linspace(-1, 1, D)
    xb = synth.f32_to_bf16_bits(x)                        # rows 0 and 5 stay zero
    q = check(xb, D, fp8.E4M3, np.float32(448.0 / np.sqrt(D)), 1.0)
    assert not q[0].any() and not q[5].any()
    d = fp8.decode(q, fp8.E4M3)
    assert np.all(d[1] == d[1, 0]) and d[2, 40] < 0 and np.count_nonzero(d[2]) == 1
    # a scale four times too large: the one-hot element saturates at -448, nothing turns into NaN
    q = check(xb, D, fp8.E4M3, np.float32(4 * 448.0 / np.sqrt(D)), 1.0)
    assert fp8.decode(q, fp8.E4M3)[2, 40] == -448.0 and np.isfinite(fp8.decode(q, fp8.E4M3)).all()


def test_qknorm_several_trips_per_workgroup():
    """More rows than one trip of the largest grid covers (2048 workgroups x 64 rows at D = 128): the pipelined
    loop runs two to four trips with a ragged last one; config 5's Q has 262144 rows."""
    rng = np.random.default_rng(11)
    rows = 3 * 131072 + 77
    xb = synth.f32_to_bf16_bits(rng.standard_normal((rows, 128)).astype(np.float32))
    check(xb, 128, fp8.E4M3, np.float32(448.0 / 5.0), 1.0)
    xb = synth.f32_to_bf16_bits(rng.standard_normal((2048 * 32 * 2 + 5, 64)).astype(np.float32))
    check(xb, 64, fp8.E5M2, np.float32(57344.0 / 5.0), 1.25)


def test_qknorm_config_shape_and_errors():
    """The Q tensor of config 3 whole ([B H S, 128] = 131072 rows), then the argument checks."""
    cfg = synth.CONFIGS[3]
    xb = synth.attention_tensors(cfg)["Q"].reshape(-1, 128)
    check(xb, 128, fp8.E4M3, np.float32(448.0 / np.sqrt(128)), 1.0)
    lib = fog.load()
    st = torch.cuda.current_stream().cuda_stream
    x = torch.zeros((4, 128), dtype=torch.int16, device="cuda")
    q = torch.zeros((4, 128), dtype=torch.uint8, device="cuda")
    f = fscalar(1.0)
    call = lib.fog_rmsnorm_quantize
    assert call(x.data_ptr(), 4, 128, 128, 1.0, 0, None, q.data_ptr(), 128, None, st) == 1
    assert call(x.data_ptr(), 4, 128, 128, 1.0, 0, f.data_ptr(), None, 128, None, st) == 1
    assert call(x.data_ptr(), 4, 128, 64, 1.0, 0, f.data_ptr(), q.data_ptr(), 128, None, st) == 2
    assert call(x.data_ptr(), -4, 128, 128, 1.0, 0, f.data_ptr(), q.data_ptr(), 128, None, st) == 2
    assert call(x.data_ptr() + 1, 4, 64, 64, 1.0, 0, f.data_ptr(), q.data_ptr(), 64, None, st) == 3
    assert call(x.data_ptr(), 4, 128, 128, 0.0, 0, f.data_ptr(), q.data_ptr(), 128, None, st) == 4
    assert call(x.data_ptr(), 4, 128, 128, 1.0, 3, f.data_ptr(), q.data_ptr(), 128, None, st) == 4
    assert call(None, 0, 128, 128, 1.0, 0, f.data_ptr(), None, 128, f.data_ptr(), st) == 0
    torch.cuda.synchronize()
    assert f.item() == 0.0                                 # the abs-max of an empty tensor is written as 0

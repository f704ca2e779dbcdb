"""GPU parity: activation kurtosis against the float64 oracle."""
import numpy as np
import pytest
import torch

from oracle import kurtosis, scaling
from paper_2505_20524_amd import fog, synth
from parity import dev

pytestmark = pytest.mark.gpu

# binary32 sums of up to 14336 terms per row and float atomics over the rows
RTOL = 2e-5


def gpu_kurt(xb, view_cols=None):
    """Runs the call twice, without and with the abs-max output; the abs-max must be bit-exact (Appendix E)."""
    x = dev(xb)
    if view_cols is not None:
        x = x[:, :view_cols]
    out = torch.full((1,), -1.0, device="cuda")
    fog.kurtosis(x, out)
    out2 = torch.full((1,), -1.0, device="cuda")
    am = torch.full((1,), -1.0, device="cuda")
    fog.kurtosis(x, out2, amax_out=am)
    view = xb if view_cols is None else xb[:, :view_cols]
    assert am.item() == scaling.amax(view)
    assert abs(out2.item() - out.item()) <= 1e-5 * abs(out.item())      # float atomics: order may differ between runs
    return out.item()


@pytest.mark.parametrize("rows,cols,pad", [(1, 8, 0), (7, 64, 0), (33, 100, 0), (64, 4096, 0), (130, 2056, 8), (5, 17, 3), (4096, 2048, 0),
                                           (5000, 14336, 0), (9, 4104, 0), (4100, 8200, 8),
                                           (4099, 1024, 0), (33, 2048, 0), (5, 512, 0), (40001, 512, 0), (17000, 1024, 8)])
def test_kurtosis_parity(rows, cols, pad):
    rng = np.random.default_rng(rows + cols)
    x = rng.standard_normal((rows, cols + pad)).astype(np.float32)
    x[:, : min(2, cols)] *= 50.0                     # outlier channels, as in the paper's activations
    xb = synth.f32_to_bf16_bits(x)
    want = kurtosis.kurt(xb[:, :cols])
    got = gpu_kurt(xb, cols if pad else None)
    assert abs(got - want) <= RTOL * want


def test_kurtosis_closed_forms_and_config_tensors():
    D = 1024
    assert gpu_kurt(synth.f32_to_bf16_bits(np.full((8, D), 1.5, np.float32))) == pytest.approx(1.0, rel=1e-6)
    oh = np.zeros((4, D), np.float32); oh[np.arange(4), [0, 7, 512, 1023]] = [2.0, -3.0, 0.5, 100.0]
    assert gpu_kurt(synth.f32_to_bf16_bits(oh)) == pytest.approx(float(D), rel=1e-6)
    z = np.zeros((4, D), np.float32); z[0, :] = 1.0
    assert gpu_kurt(synth.f32_to_bf16_bits(z)) == pytest.approx(0.25, rel=1e-6)     # zero rows contribute 0
    out = torch.full((1,), -1.0, device="cuda")
    assert fog.load().fog_kurtosis(None, 0, 64, 64, out.data_ptr(), None, torch.cuda.current_stream().cuda_stream) == 0
    torch.cuda.synchronize()
    assert out.item() == 0.0
    # the activations of config 1 (4 outlier channels x50) and config 5 (2 channels x1000, "massive activations")
    for cid in (1, 5):
        xb = synth.linear_tensors(synth.CONFIGS[cid], 0, want=("X",))["X"]
        want = kurtosis.kurt(xb)
        assert abs(gpu_kurt(xb) - want) <= RTOL * want
        assert want > (50 if cid == 1 else 1500)     # far above the Gaussian 3: what the diagnostic is for


def test_kurtosis_argument_errors():
    lib = fog.load()
    st = torch.cuda.current_stream().cuda_stream
    x = torch.zeros(64, dtype=torch.int16, device="cuda")
    out = torch.zeros(1, device="cuda")
    assert lib.fog_kurtosis(x.data_ptr(), 4, 16, 16, None, None, st) == 1
    assert lib.fog_kurtosis(x.data_ptr(), -1, 16, 16, out.data_ptr(), None, st) == 2
    assert lib.fog_kurtosis(x.data_ptr(), 4, 16, 8, out.data_ptr(), None, st) == 2
    assert lib.fog_kurtosis(x.data_ptr() + 1, 4, 8, 8, out.data_ptr(), None, st) == 3
    assert lib.fog_kurtosis(None, 4, 16, 16, out.data_ptr(), None, st) == 1

"""Pins for the oracle's kurtosis (CPU only)."""
import numpy as np
import scipy.stats

from oracle import kurtosis
from paper_2505_20524_amd import synth


def bits(x):
    return synth.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def test_closed_forms():
    D = 64
    assert kurtosis.kurt(bits(np.full((3, D), 2.5))) == 1.0                 # constant vector
    one_hot = np.zeros((2, D)); one_hot[0, 5] = 3.0; one_hot[1, 63] = -0.5
    assert kurtosis.kurt(bits(one_hot)) == float(D)                          # a single outlier: the maximum, D
    two = np.zeros((1, D)); two[0, :2] = [1.0, -1.0]
    assert kurtosis.kurt(bits(two)) == D / 2
    assert kurtosis.kurt(bits(np.zeros((4, D)))) == 0.0                      # all-zero rows contribute 0
    mixed = np.vstack([np.full((1, D), 1.0), one_hot[:1]])
    assert kurtosis.kurt(bits(mixed)) == (1.0 + D) / 2                       # tensor value = mean over token vectors
    assert kurtosis.kurt(np.zeros((0, D), np.uint16)) == 0.0


def test_invariances_and_growth_with_outlier():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((16, 256)).astype(np.float32)
    xb = bits(x)
    k = kurtosis.kurt_rows(xb)
    assert np.allclose(kurtosis.kurt_rows(bits(synth.bf16_bits_to_f32(xb) * 4.0)), k, rtol=1e-12)   # scale (power of two: exact in bf16)
    assert np.allclose(kurtosis.kurt_rows(xb ^ np.uint16(0x8000)), k, rtol=1e-15)                     # sign
    perm = rng.permutation(256)
    assert np.allclose(kurtosis.kurt_rows(xb[:, perm]), k, rtol=1e-12)                                # order of features
    prev = None
    for tau in (4, 16, 64, 256):                       # the larger the outlier, the larger the kurtosis (Section 4)
        y = x.copy(); y[:, 0] = tau
        v = kurtosis.kurt(bits(y))
        assert prev is None or v > prev
        prev = v
    assert prev > 200                                  # approaches D = 256


def test_against_library_kurtosis_on_symmetrised_data():
    """For data with exactly zero mean the un-centred definition is Pearson's kurtosis."""
    rng = np.random.default_rng(1)
    x = synth.bf16_bits_to_f32(bits(rng.standard_normal((8, 512)) * np.exp(rng.standard_normal((8, 512)))))
    sym = np.concatenate([x, -x], axis=1)
    lib = scipy.stats.kurtosis(sym.astype(np.float64), axis=1, fisher=False, bias=True)
    assert np.allclose(kurtosis.kurt_rows(bits(sym)), lib, rtol=1e-12)
    g = kurtosis.kurt(bits(rng.standard_normal((64, 8192))))
    assert abs(g - 3.0) < 0.05                          # Gaussian data: 3

"""Activation kurtosis, the paper's outlier diagnostic (Section 4).

For a token vector x in R^D:  kurt(x) = mu[x^4] / (mu[x^2])^2, element-wise powers, no centring
(the paper stresses that x is not shifted to zero mean); for a tensor of N x C token vectors,
kurt(X) is the average over the N C vectors.

Reading of a garbled formula: the paper prints the denominator as sigma^2[x^2] and calls sigma^2
"the sample variance".  Taken literally (variance of x^2) the quantity would FALL towards 1 as an
outlier grows, against the text's "maximized when few elements reach extremely large values".
The reading taken here is the squared un-centred second moment, (mu[x^2])^2, which is the
definition of the work the paper cites for it; it gives 1 for a constant vector, D for a one-hot
vector and 3 for Gaussian data.  A vector of zeros contributes 0 to the average.
"""
import numpy as np

from . import bf16


def kurt_rows(x_bits):
    """Per-row kurtosis of a bf16 matrix [rows, D] (uint16 bit patterns) as float64 [rows]."""
    x = bf16.bits_to_f64(np.asarray(x_bits, dtype=np.uint16))
    m2 = np.mean(x ** 2, axis=-1)
    m4 = np.mean(x ** 4, axis=-1)
    with np.errstate(divide="ignore", invalid="ignore"):
        k = m4 / (m2 * m2)
    return np.where(m2 > 0, k, 0.0)


def kurt(x_bits):
    """kurt(X): the mean of the per-token kurtosis."""
    k = kurt_rows(x_bits)
    return float(k.mean()) if k.size else 0.0

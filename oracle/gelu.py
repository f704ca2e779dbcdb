"""GeLU and tanh_alpha activations fused with the FP8 cast (Section 3, table of the architecture suite; cast of Appendix E).

Test infrastructure only.  Two of the FOG variants use GeLU between the feed-forward GEMMs, and the
FOG-flash variant regularises queries and keys with tanh_alpha(x) = tanh(alpha x) (Section 3).  The
paper names GeLU without a formula; it is read as the original definition
    GeLU(x) = x Phi(x),    Phi the standard normal distribution function,
not the tanh approximation.  Both activations feed an FP8 cast:
    y = f(x),   q = FP8cast(rho * y)   (rho * y rounded once to binary32, then to the FP8 grid),
    amax = max |y|.
y is not a stored tensor: the code is a rounding decision on a value the device computes in
binary32, so `*_window` gives the codes at both ends of a relative window, the set of valid results.
"""
import numpy as np
from scipy import special

from . import bf16, fp8


def gelu(x):
    """x Phi(x) in float64; Phi(x) = erfc(-x / sqrt 2) / 2 keeps full relative accuracy in the negative tail."""
    x = np.asarray(x, dtype=np.float64)
    return 0.5 * x * special.erfc(-x / np.sqrt(2.0))


def tanh_alpha(x, alpha):
    return np.tanh(np.float64(alpha) * np.asarray(x, dtype=np.float64))


def _cast(y, rho, fmt):
    return fp8.encode_sat((np.float64(np.float32(rho)) * y).astype(np.float32), fmt)


def gelu_amax(x_bits):
    y = gelu(bf16.bits_to_f64(np.asarray(x_bits, dtype=np.uint16)))
    return float(np.abs(y).max()) if y.size else 0.0


def gelu_quantize(x_bits, rho, fmt):
    return _cast(gelu(bf16.bits_to_f64(np.asarray(x_bits, dtype=np.uint16))), rho, fmt)


def gelu_window(x_bits, rho, fmt, rel=2.0 ** -19):
    """(code_lo, code_hi).  The relative window grows with x^2 on the negative side: there Phi(x) has the
    relative condition number x^2 (d log Phi / d log x -> -x^2), so the binary32 rounding of the argument
    alone moves the value by x^2 2^-24."""
    x = bf16.bits_to_f64(np.asarray(x_bits, dtype=np.uint16))
    r = rel + np.where(x < 0, x * x, 0.0) * 2.0 ** -23
    y = gelu(x)
    return _cast(y * (1.0 - r), rho, fmt), _cast(y * (1.0 + r), rho, fmt)


def tanh_amax(x_bits, alpha):
    y = tanh_alpha(bf16.bits_to_f64(np.asarray(x_bits, dtype=np.uint16)), alpha)
    return float(np.abs(y).max()) if y.size else 0.0


def tanh_quantize(x_bits, rho, fmt, alpha):
    return _cast(tanh_alpha(bf16.bits_to_f64(np.asarray(x_bits, dtype=np.uint16)), alpha), rho, fmt)


def tanh_window(x_bits, rho, fmt, alpha, rel=2.0 ** -19):
    y = tanh_alpha(bf16.bits_to_f64(np.asarray(x_bits, dtype=np.uint16)), alpha)
    return _cast(y * (1.0 - rel), rho, fmt), _cast(y * (1.0 + rel), rho, fmt)

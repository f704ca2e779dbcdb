"""xIELU activation fused with the FP8 cast (Appendix B of the paper, equation xIELU; cast of Appendix E).

The FOG-max variant uses, element-wise,
    xIELU(x) = alpha_p x^2 + 0.5 x                          for x > 0,
               alpha_n (e^x - 1) - alpha_n x + 0.5 x        for x <= 0,
with alpha_p and alpha_n trainable scalars of the layer (given here as plain numbers; how the
cited work parametrises them for training is outside the paper's equation and not modelled).
The activation sits between the two GEMMs of the feed-forward block, so its output is what gets
cast to FP8 for the second GEMM:
    y = xIELU(x),   q = FP8cast(rho * y)   (rho * y rounded once to binary32, then to the FP8 grid),
    amax = max |y|  (for the history of delayed scaling).
y is not a stored tensor: the code is a rounding decision on a value the device computes in
binary32 (expm1, a few multiplies and adds); `quantize_window` gives the codes at both ends of a
relative window, the set of valid results of each element.
"""
import numpy as np

from . import bf16, fp8


def xielu(x, alpha_p, alpha_n):
    """The paper's equation on float64 values."""
    x = np.asarray(x, dtype=np.float64)
    ap, an = np.float64(alpha_p), np.float64(alpha_n)
    pos = ap * x * x + 0.5 * x
    neg = an * np.expm1(np.minimum(x, 0.0)) - an * x + 0.5 * x
    return np.where(x > 0, pos, neg)


def activate(x_bits, alpha_p, alpha_n):
    return xielu(bf16.bits_to_f64(np.asarray(x_bits, dtype=np.uint16)), alpha_p, alpha_n)


def amax(x_bits, alpha_p, alpha_n):
    y = activate(x_bits, alpha_p, alpha_n)
    return float(np.abs(y).max()) if y.size else 0.0


def quantize(x_bits, rho, fmt, alpha_p, alpha_n):
    t = (np.float64(np.float32(rho)) * activate(x_bits, alpha_p, alpha_n)).astype(np.float32)
    return fp8.encode_sat(t, fmt)


def quantize_window(x_bits, rho, fmt, alpha_p, alpha_n, rel=2.0 ** -19):
    """(code_lo, code_hi): the casts of rho * y * (1 -+ rel)."""
    y = np.float64(np.float32(rho)) * activate(x_bits, alpha_p, alpha_n)
    lo = fp8.encode_sat((y * (1.0 - rel)).astype(np.float32), fmt)
    hi = fp8.encode_sat((y * (1.0 + rel)).astype(np.float32), fmt)
    return lo, hi

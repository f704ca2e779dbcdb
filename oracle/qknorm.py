"""QK RMS normalisation with frozen gains, fused with the FP8 cast (Section 3; Appendix A).

Section 3 defines the entropy-regularising block of the attention as
    N_gamma(x) = gamma (.) x / rms(x),      rms(x) = ||x||_2 / sqrt(D),
applied to every query and key vector x in R^D (one head of one token).  The FOG variants freeze
the gains (Table of Section 3, entries marked "not trainable"), and Appendix A folds the frozen
value gamma_0 into the softmax scale (s = gamma_0^2 / sqrt(D_qk)); what is left in front of the
FP8 attention is x / rms(x) times one scalar.  The function below is that producer written out
together with the cast of Appendix E that consumes it:
    y = gain * x / rms(x)            (float64 here)
    q = FP8cast(rho * y)             (rho * y rounded once to binary32, then to the FP8 grid)
    amax = max |y|                   (for the history of delayed scaling)
The paper's formula has no epsilon: a vector of zeros has rms 0 and is mapped to zeros.

Because y is not a stored tensor, the code q is a rounding decision taken on a value that the
device computes in binary32 (sum of D squares, square root, division): `quantize_window` returns
the two codes obtained at the ends of a relative window around rho * y; an element whose two
codes differ has two valid results, every other element exactly one.
"""
import numpy as np

from . import bf16, fp8


def normalize(x_bits, gain=1.0):
    """y = gain * x / rms(x) per row of a bf16 matrix [rows, D]; float64 [rows, D]."""
    x = bf16.bits_to_f64(np.asarray(x_bits, dtype=np.uint16))
    ms = np.mean(x * x, axis=-1, keepdims=True)
    with np.errstate(divide="ignore", invalid="ignore"):
        y = np.float64(gain) * x / np.sqrt(ms)
    return np.where(ms > 0, y, 0.0)


def amax(x_bits, gain=1.0):
    y = normalize(x_bits, gain)
    return float(np.abs(y).max()) if y.size else 0.0


def quantize(x_bits, rho, fmt, gain=1.0):
    """FP8 codes of rho * normalize(x): one binary32 rounding of the product, then the saturating cast."""
    t = (np.float64(np.float32(rho)) * normalize(x_bits, gain)).astype(np.float32)
    return fp8.encode_sat(t, fmt)


def quantize_window(x_bits, rho, fmt, gain=1.0, rel=2.0 ** -20):
    """(code_lo, code_hi): the casts of rho * y * (1 -+ rel), the set of valid codes of each element."""
    y = np.float64(np.float32(rho)) * normalize(x_bits, gain)
    lo = fp8.encode_sat((y * (1.0 - rel)).astype(np.float32), fmt)
    hi = fp8.encode_sat((y * (1.0 + rel)).astype(np.float32), fmt)
    return lo, hi

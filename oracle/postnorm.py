"""Post-RMSNorm with its residual connection, fused with the FP8 cast of the sum (Section 3; cast of Appendix E).

Test infrastructure only.  The FOG block has no pre-normalisation; each sub-layer's output y (attention
or feed-forward) goes through an RMSNorm with a trainable gains vector before the residual connection
(Section 3: post-normalised architecture, gains initialised to 1/sqrt(num_layers)):
    x_new = x + N_gamma(y),      N_gamma(y) = gamma (.) y / rms(y),   rms(y) = ||y||_2 / sqrt(D).
x_new is the residual stream: it is stored (bf16) and, with no pre-norm in between, it is also the
input of the next sub-layer's first GEMM, i.e. the tensor that gets cast to FP8:
    x_new_bf16 = bf16(x_new),   q = FP8cast(rho * x_new_bf16),   amax = max |x_new_bf16|.
The formula has no epsilon: a zero vector y adds nothing.

The sum is evaluated by the device in binary32 and rounded once to bf16; `residual_window` returns the
bf16 values at both ends of the interval that evaluation can land in.  The FP8 codes and the abs-max are
then exact functions of the bf16 tensor that was actually stored (the per-tensor cast oracle applies).
"""
import numpy as np

from . import bf16


def normalize(y_bits, gamma):
    """gamma (.) y / rms(y) per row; float64 [rows, D].  gamma: [D] binary32 values."""
    y = bf16.bits_to_f64(np.asarray(y_bits, dtype=np.uint16))
    g = np.asarray(gamma, dtype=np.float32).astype(np.float64)
    ms = np.mean(y * y, axis=-1, keepdims=True)
    with np.errstate(divide="ignore", invalid="ignore"):
        n = g * y / np.sqrt(ms)
    return np.where(ms > 0, n, 0.0)


def residual(x_bits, y_bits, gamma):
    """x + N_gamma(y) in float64."""
    return bf16.bits_to_f64(np.asarray(x_bits, dtype=np.uint16)) + normalize(y_bits, gamma)


def residual_bf16(x_bits, y_bits, gamma):
    return bf16.f64_to_bits_rne(residual(x_bits, y_bits, gamma))


def residual_window(x_bits, y_bits, gamma, rel_norm=2.0 ** -20, rel_sum=2.0 ** -23):
    """(bits_lo, bits_hi): bf16 roundings of the ends of x_new -+ (rel_norm |N(y)| + rel_sum |x_new|).
    rel_norm covers the binary32 sum of squares, square root, division and gain product, rel_sum the
    rounding of the final addition."""
    n = normalize(y_bits, gamma)
    s = bf16.bits_to_f64(np.asarray(x_bits, dtype=np.uint16)) + n
    w = rel_norm * np.abs(n) + rel_sum * np.abs(s)
    return bf16.f64_to_bits_rne(s - w), bf16.f64_to_bits_rne(s + w)

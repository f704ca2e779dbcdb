"""Per-tensor scaling: abs-max, scale, cast (with optional transpose), amax history.

Appendix E defines the scale of a tensor as rho = FP8MaxValue / (2^m * max H)
with H a history of abs-max values (just-in-time scaling, Section 2, is the
history of length one holding the tensor's own abs-max), the history update
H <- {max|x|} U {h_t, t >= 2}, and the cast as FP8cast(rho * X).  Appendix C
states the same scale as MaxFP8Value / absmax(x).

Readings where the paper is silent: the scale is a binary32 number obtained by
one correctly rounded binary32 division; rho = 1 when the abs-max is zero or
not finite; rho is capped at the largest finite binary32; the product rho * x is
rounded to binary32 once before the FP8 rounding.
"""
import numpy as np

from . import bf16, fp8

_FLT_MAX = np.float32(3.4028234663852886e38)


def amax(x_bits):
    """max_i |x_i| of a bf16 tensor (given as uint16 bit patterns), as float32 (exact)."""
    b = np.asarray(x_bits, dtype=np.uint16)
    if b.size == 0:
        return np.float32(0.0)
    return np.float32(np.max(np.abs(bf16.bits_to_f32(b))))


def compute_scale(amax_value, fmt, margin=0):
    """(rho, 1/rho) as float32 from an abs-max: rho = fl32(FP8MaxValue / (2^margin * amax))."""
    a = np.float32(amax_value)
    if not np.isfinite(a) or a == 0:
        rho = np.float32(1.0)
    else:
        with np.errstate(over="ignore", divide="ignore"):
            denom = np.float32(a * np.float32(2.0 ** margin))
            rho = np.float32(np.float32(fp8.fp8_max(fmt)) / denom)
        if not np.isfinite(rho):
            rho = _FLT_MAX
        if rho == 0:
            rho = np.float32(1.0)
    with np.errstate(over="ignore"):
        rho_inv = np.float32(np.float32(1.0) / rho)
    return rho, rho_inv


def quantize(x_bits, rho, fmt):
    """FP8cast(rho * X): codes of encode_sat(fl32(float(x) * rho)), same shape as x."""
    x = bf16.bits_to_f32(np.asarray(x_bits, dtype=np.uint16))
    with np.errstate(over="ignore", under="ignore"):
        t = (x * np.float32(rho)).astype(np.float32)     # one binary32 rounding
    return fp8.encode_sat(t, fmt)


def quantize_with_transpose(x_bits, rho, fmt):
    """(q, qT): the cast of a 2-D tensor and the same codes laid out transposed."""
    q = quantize(x_bits, rho, fmt)
    return q, np.ascontiguousarray(q.T)


def history_scale(history, fmt, margin=0):
    """Delayed scaling: rho from the maximum of the abs-max history (Appendix E)."""
    h = np.asarray(history, dtype=np.float32)
    return compute_scale(np.float32(h.max()) if h.size else np.float32(0), fmt, margin)


def history_update(history, new_amax):
    """H <- {amax(X)} U {h_t}_{t>=2}: newest value replaces the first entry after a roll.

    The history is kept newest-first; the oldest entry (the last) falls out.
    """
    h = np.asarray(history, dtype=np.float32)
    out = np.empty_like(h)
    out[0] = np.float32(new_amax)
    out[1:] = h[:-1]
    return out

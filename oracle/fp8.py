"""OCP 8-bit floating point: E4M3 and E5M2 decode and saturating encode.

Section 2 of the paper names the two formats (four exponent + three mantissa
bits for forward tensors, five + two for backward tensors) and refers to the
OCP FP8 definition for the rest.  The constants below are that definition:

  E4M3: bias 7, no infinities, NaN = S.1111.111, max finite 448 (0x7E),
        min normal 2^-6, subnormals k * 2^-9 (k = 1..7).
  E5M2: bias 15, IEEE-like: inf = S.11111.00, NaN = S.11111.{01,10,11},
        max finite 57344 (0x7B), min normal 2^-14, subnormals k * 2^-16.

`decode` is the closed form.  `encode_sat` is round-to-nearest-even onto the
format's grid with saturation to the largest finite value (the cast used
before every FP8 GEMM, Appendix E: FP8cast(rho * X)), done by integer
manipulation of the binary32 bit pattern.  It is pinned in the tests against a
brute-force nearest-code search, against every midpoint, and against
independent library casts.
"""
import numpy as np

E4M3 = 0
E5M2 = 1

# (mantissa bits, exponent bias, minimum normal exponent, largest finite value, its code)
_FMT = {
    E4M3: dict(mbits=3, bias=7, emin=-6, fmax=448.0, cmax=0x7E, name="E4M3"),
    E5M2: dict(mbits=2, bias=15, emin=-14, fmax=57344.0, cmax=0x7B, name="E5M2"),
}


def fp8_max(fmt):
    """Largest finite magnitude of the format (the paper's FP8MaxValue, Appendix E)."""
    return _FMT[fmt]["fmax"]


def decode(codes, fmt):
    """uint8 codes -> float64 values (exact).  NaN and infinity codes decode to nan / inf."""
    f = _FMT[fmt]
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    mb, bias = f["mbits"], f["bias"]
    sign = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> mb) & ((1 << (7 - mb)) - 1)
    m = c & ((1 << mb) - 1)
    sub = m.astype(np.float64) * 2.0 ** (1 - bias - mb)
    nor = (1.0 + m.astype(np.float64) / (1 << mb)) * np.exp2((e - bias).astype(np.float64))
    v = np.where(e == 0, sub, nor)
    if fmt == E4M3:
        v = np.where((c & 0x7F) == 0x7F, np.nan, v)
    else:
        v = np.where(e == 31, np.where(m == 0, np.inf, np.nan), v)
    return sign * v


def encode_sat(t, fmt):
    """binary32 values -> uint8 codes: round to nearest, ties to even mantissa, saturating.

    NaN -> 0x7F | sign.  |t| >= FP8MaxValue (infinities included) -> the largest
    finite code with t's sign.  A magnitude exactly halfway between zero and the
    smallest subnormal goes to zero; the sign of zero is kept.
    """
    f = _FMT[fmt]
    mb, bias, emin = f["mbits"], f["bias"], f["emin"]
    t = np.ascontiguousarray(t, dtype=np.float32)
    bits = t.view(np.uint32).astype(np.int64)
    sign = (bits >> 24) & 0x80
    a = bits & 0x7FFFFFFF
    isnan = a > 0x7F800000
    exp32 = a >> 23
    man = a & 0x7FFFFF
    # binary32 subnormals are far below half the smallest FP8 subnormal: they round to zero.
    E = exp32 - 127                       # unbiased exponent of the binary32 value
    sig = np.where(exp32 > 0, man | 0x800000, 0)   # 24-bit significand, value = sig * 2^(E-23)
    e = np.maximum(E, emin)               # exponent of the FP8 binade the result is rounded in
    shift = np.minimum((23 - mb) + (e - E), 40)    # low bits of sig that fall below the FP8 quantum
    n = sig >> shift
    rem = sig & ((np.int64(1) << shift) - 1)
    half = np.int64(1) << (shift - 1)
    up = (rem > half) | ((rem == half) & ((n & 1) == 1))
    n = n + up
    # n = 2^(mb+1) carries into the next binade; subnormals (n < 2^mb at e = emin) give code n.
    code = ((e + bias) << mb) + n - (1 << mb)
    big = a >= np.float32(f["fmax"]).view(np.uint32).astype(np.int64)
    code = np.where(big, f["cmax"], code)
    code = np.where(isnan, 0x7F, code)
    return (code | sign).astype(np.uint8)

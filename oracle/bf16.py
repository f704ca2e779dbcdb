"""bfloat16 <-> float plumbing for the oracle (format handling, no method arithmetic).

bfloat16 is the upper 16 bits of IEEE binary32 (1 sign, 8 exponent, 7 mantissa
bits).  The FP8 GEMM "returns the BF16 result" (Appendix E, end-to-end GEMM
equation), so the oracle needs an exact float64 -> bf16 round-to-nearest-even
to state results in the output format.
"""
import numpy as np


def bits_to_f32(bits):
    """uint16 bf16 bit patterns -> float32 (exact)."""
    b = np.asarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bits_to_f64(bits):
    return bits_to_f32(bits).astype(np.float64)


def f64_to_bits_rne(v):
    """float64 -> bf16 bit pattern with ONE round-to-nearest-even (no trip through binary32).

    bf16 keeps 8 significant bits; normal exponents are those of binary32
    (min normal 2^-126, subnormal quantum 2^-133); overflow goes to infinity.
    """
    v = np.asarray(v, dtype=np.float64)
    a = np.abs(v)
    sign = (np.signbit(v)).astype(np.uint16) << np.uint16(15)
    out = np.zeros(v.shape, dtype=np.uint16)
    nan = np.isnan(v)
    fin = np.isfinite(v) & (a > 0)
    m, e = np.frexp(np.where(fin, a, 1.0))          # a = m * 2^e, m in [0.5, 1)
    E = e - 1                                        # a in [2^E, 2^(E+1))
    Eq = np.maximum(E, -126)
    q = np.ldexp(1.0, Eq - 7)                        # spacing of bf16 in that binade
    n = np.rint(np.where(fin, a, 0.0) / q)           # exact division by a power of two; rint is RNE
    # n in [0, 256]; 256 carries into the next binade, which the formula below does by itself
    code = ((Eq + 127).astype(np.int64) << 7) + n.astype(np.int64) - 128
    code = np.where(fin, code, 0)
    code = np.where(code >= 0x7F80, 0x7F80, code)    # overflow -> inf
    out = code.astype(np.uint16)
    out = np.where(np.isinf(v), np.uint16(0x7F80), out)
    out = np.where(nan, np.uint16(0x7FC0), out)
    return (out | sign).astype(np.uint16)


def f64_round(v):
    """float64 -> nearest bf16 value, returned as float64."""
    return bits_to_f64(f64_to_bits_rne(v))


def half_ulp(v):
    """Half the bf16 spacing at |v| (float64): the error any bf16 result may carry."""
    a = np.abs(np.asarray(v, dtype=np.float64))
    _, e = np.frexp(np.where(a > 0, a, 1.0))
    Eq = np.maximum(e - 1, -126)
    return np.ldexp(1.0, Eq - 8)

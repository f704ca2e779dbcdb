"""Helpers shared by the GPU parity tests: device upload and the output gates.

Gate for bf16 outputs (GEMM, attention).  The library rounds its binary32 result once to
bfloat16; half a bf16 spacing is 2^-8 of the value's binade, i.e. up to 3.9e-3 relative, so a
2e-3 bound cannot be asked of the ROUNDED value against a float64 oracle.  The 2e-3 is taken
as a bound on the error BEFORE that final rounding, normalised by the tensor's largest
magnitude:  |v - oracle| <= rel * max|oracle|  with y = bf16(v).  Because rounding is monotone
this is checked exactly on the rounded output:  bf16(oracle - tol) <= y <= bf16(oracle + tol).
For attention the casts of P and dS are rounding decisions the kernel takes in binary32 on
matrix-instruction results.  The FP8 matrix instruction aligns the eight products of a group to
the group's largest exponent and drops bits more than 13 places below it (measured on the device
with cancelling operands); the oracle bounds that truncation per score, and an element whose
pre-cast value can cross a rounding boundary inside the bound has two valid codes.  The gate is
widened by exactly the linear effect of those elements (`slack`, computed by the oracle).
A second, much tighter statistic is reported and bounded as well: the fraction of elements
whose bf16 code differs from bf16(oracle), and by how many bf16 steps.
"""
import numpy as np
import torch

from oracle import bf16

REL = 2e-3


def dev(a):
    """numpy array -> CUDA tensor with the same bytes (uint16 travels as int16)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    return torch.from_numpy(a).cuda()


def host_u16(t):
    return t.cpu().numpy().view(np.uint16)


def fscalar(v):
    return torch.tensor([float(v)], dtype=torch.float32, device="cuda")


def ordered(bits):
    """bf16 bit patterns -> integers ordered like the values (for step counting)."""
    b = bits.astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)


def check_bf16(y_bits, oracle64, rel=REL, what="", max_flip_frac=0.02, slack=None):
    oracle64 = np.asarray(oracle64, dtype=np.float64)
    y = bf16.bits_to_f64(y_bits)
    assert np.all(np.isfinite(y)), what + ": non-finite output"
    scale = np.abs(oracle64).max()
    tol = rel * scale
    if slack is not None:                 # valid-result set of ambiguous rounding decisions (attention casts)
        tol = tol + np.asarray(slack, dtype=np.float64)
    lo = bf16.f64_round(oracle64 - tol)
    hi = bf16.f64_round(oracle64 + tol)
    bad = (y < lo) | (y > hi)
    err = np.abs(y - oracle64).max() / scale if scale > 0 else 0.0
    assert not bad.any(), "%s: %d of %d elements outside the %.0e gate (max normalised error %.3e)" % (
        what, int(bad.sum()), bad.size, rel, err)
    ref_bits = bf16.f64_to_bits_rne(oracle64)
    steps = np.abs(ordered(np.asarray(y_bits)) - ordered(ref_bits))
    big = np.abs(oracle64) >= scale * 2.0 ** -6
    flips = float((steps[big] > 0).mean()) if big.any() else 0.0
    worst = int(steps[big].max()) if big.any() else 0
    assert flips <= max_flip_frac, "%s: %.3f%% of elements differ from bf16(oracle)" % (what, 100 * flips)
    return dict(max_norm_err=float(err), flip_frac=flips, max_steps=worst)

"""Helpers shared by the GPU parity tests: device upload and the output gates.

Gate for bf16 outputs (GEMM, attention).  The library rounds its binary32 result once to
bfloat16; half a bf16 spacing is 2^-8 of the value's binade, i.e. up to 3.9e-3 relative, so a
2e-3 bound cannot be asked of the ROUNDED value against a float64 oracle.  The 2e-3 is taken
as a bound on the error BEFORE that final rounding, normalised by the tensor's largest
magnitude:  |v - oracle| <= rel * max|oracle|  with y = bf16(v).  Because rounding is monotone
this is checked exactly on the rounded output:  bf16(oracle - tol) <= y <= bf16(oracle + tol).
A second, much tighter statistic is bounded as well: the fraction of elements whose bf16 code
differs from bf16(oracle), and by how many bf16 steps.

Attention (`check_attention`).  The casts of P and dS are rounding decisions the kernel takes in
binary32 on matrix-instruction results, the oracle in float64; an element whose pre-cast value lies
within the instruction's truncation of a rounding boundary has two valid codes (tests/mfma_model.py,
pinned on the device by tests/test_gpu_mfma_model.py).  The element-wise gate is widened by exactly the
linear effect of those elements (`slack`) -- a worst-case sum, so on its own it would let a real defect
of a few gate-widths through on some elements.  Four statistics, which a defect of that kind moves and
legitimate code flips (few, zero-mean) do not, are therefore bounded too, with bounds frozen from
measurement (a few times what the kernels show, far below what the slack alone would admit):
  * the fraction of elements outside the PLAIN gate (no slack),
  * the RMS error normalised by the tensor's largest magnitude,
  * the median slack in units of the plain gate (the slack must stay a correction, not the gate),
  * the fraction of large elements whose bf16 code differs from bf16(oracle).
Every call appends its figures to STATS; the GPU run prints them at the end (tests/conftest.py).
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


def check_gemm_elementwise(y_bits, oracle64, absdot64, what=""):
    """Element-wise companion of the tensor-normalised gate, for GEMM outputs: every element, however small against the
    tensor's maximum, must lie within half a bf16 step of its own oracle value plus what the accumulation can lose on THAT
    element: 2^-12 of sum_k |a||b| (the matrix instruction keeps 13 places below the largest product of a group of eight;
    binary32 adds of the group sums lose far less).  absdot64 = sinv_a sinv_b (|decode(A)| x |decode(B)|)."""
    oracle64 = np.asarray(oracle64, dtype=np.float64)
    y = bf16.bits_to_f64(y_bits)
    tol = 2.0 ** -12 * np.asarray(absdot64, dtype=np.float64)
    lo = bf16.f64_round(oracle64 - tol)
    hi = bf16.f64_round(oracle64 + tol)
    bad = (y < lo) | (y > hi)
    assert not bad.any(), "%s: %d of %d elements outside their own half-step + accumulation bound" % (what, int(bad.sum()), bad.size)


STATS = []     # one line per attention check: printed by the terminal summary of a GPU run

# Bounds of the four statistics, frozen from measurement over every attention check of the GPU suite (290 checked
# tensors: small shapes, grouped queries, 8192 / 16384 tokens, configs 3, 4 and 5).  Measured maxima in brackets.
FULL_HEAD = 262144            # elements of one (batch, head) pair at 2048 tokens: the benchmark configs' sizes
MAX_EXCEED_FRAC_FULL = 0.005  # outside the plain gate, full heads         [0.0024: config 4, Student-t; N(0,1) configs 0.00014]
MAX_EXCEED_FRAC = 0.01        # ... shorter sequences                      [0.0049]
MAX_RMS_FULL = 6e-4           # normalised RMS error, full heads           [3.5e-4]
MAX_RMS_SMALL = 2e-3          # ... shorter sequences: one flipped E5M2 code of dS (a 2^-2 step) weighs more   [1.4e-3]
MAX_MEDIAN_SLACK_FULL = 1.0   # median slack in gate widths, full heads    [0.95]
MAX_MEDIAN_SLACK_SMALL = 8.0  # ... shorter sequences, grouped queries (slacks of a group add up)             [6.8]
MAX_FLIP_FRAC = 0.2           # large elements whose bf16 code differs from bf16(oracle)                      [0.144]


def check_attention(y_bits, oracle64, slack, what="", rel=REL, max_exceed_frac=None, max_rms=None,
                    max_median_slack=None, max_flip_frac=MAX_FLIP_FRAC):
    """The slack-widened element-wise gate plus the four bounded statistics described in the module header."""
    oracle64 = np.asarray(oracle64, dtype=np.float64)
    slack = np.broadcast_to(np.asarray(slack, dtype=np.float64), oracle64.shape)
    full = oracle64.size >= FULL_HEAD
    if max_exceed_frac is None:
        max_exceed_frac = MAX_EXCEED_FRAC_FULL if full else MAX_EXCEED_FRAC
    if max_rms is None:
        max_rms = MAX_RMS_FULL if full else MAX_RMS_SMALL
    if max_median_slack is None:
        max_median_slack = MAX_MEDIAN_SLACK_FULL if full else MAX_MEDIAN_SLACK_SMALL
    st = check_bf16(y_bits, oracle64, rel=rel, what=what, max_flip_frac=1.0, slack=slack)
    y = bf16.bits_to_f64(y_bits)
    scale = np.abs(oracle64).max()
    gate = rel * scale
    plain_bad = (y < bf16.f64_round(oracle64 - gate)) | (y > bf16.f64_round(oracle64 + gate))
    exceed = float(plain_bad.mean())
    rms = float(np.sqrt(np.mean((y - oracle64) ** 2)) / scale) if scale > 0 else 0.0
    med = float(np.median(slack) / gate) if gate > 0 else 0.0
    worst_used = float(np.max(np.where(plain_bad, np.abs(y - oracle64), 0.0)) / gate) if gate > 0 else 0.0
    STATS.append("%-18s n=%-8d outside plain gate %.4f%%  rms %.2e  median slack %.2f gate  max slack %.1f gate  "
                 "largest error %.2f gate  bf16 flips %.3f" % (what, oracle64.size, 100 * exceed, rms, med,
                                                             float(slack.max() / gate) if gate > 0 else 0.0, worst_used,
                                                             st["flip_frac"]))
    assert exceed <= max_exceed_frac, "%s: %.3f%% of elements outside the plain %.0e gate (bound %.3f%%)" % (
        what, 100 * exceed, rel, 100 * max_exceed_frac)
    assert rms <= max_rms, "%s: normalised RMS error %.2e above %.1e" % (what, rms, max_rms)
    assert med <= max_median_slack, "%s: median slack is %.2f gate widths" % (what, med)
    assert st["flip_frac"] <= max_flip_frac, "%s: %.1f%% of large elements differ from bf16(oracle)" % (what, 100 * st["flip_frac"])
    return dict(st, exceed_frac=exceed, rms=rms, median_slack=med)

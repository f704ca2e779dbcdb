"""GPU pin of the device facts that tests/mfma_model.py rests on, measured through the C ABI (fog_fp8_gemm).

The FP8 matrix instruction does not sum its products exactly.  What the attention parity gate assumes
about it (mfma_model.MFMA_GROUP, MFMA_KEEP_BITS) is measured here on every GPU run, with cancelling
operands: a contraction row holds +B and -B (two products that cancel exactly) and one small product
2^k below |B|.  The exact result is the small product; whatever the instruction dropped while aligning it
to B shows in the output (a power of two or a few-bit value: exact in bf16, so the rounding of the result
hides nothing).  Three statements are checked:
  (1) small and B in the SAME group of eight consecutive contraction indices, k <= MFMA_KEEP_BITS:
      the small product survives exactly (the bound in mfma_model assumes at least that many kept places);
  (2) small in a DIFFERENT aligned group of eight than both +B and -B: exact for every k tried (the
      alignment is per group of eight, not wider, which is what makes the per-group bound valid);
  (3) same group, any k, few-bit small products: the loss never exceeds mfma_model.dot_uncertainty.
And one descriptive statement, so that the model is known not to be vacuous on this part:
  (4) same group, k >= 16: the small product vanishes altogether.
"""
import numpy as np
import pytest
import torch

from oracle import fp8
from paper_2505_20524_amd import fog
import mfma_model
from parity import dev, fscalar, host_u16

pytestmark = pytest.mark.gpu


def e4m3_of(v):
    """Code of an exactly representable value."""
    c = fp8.encode_sat(np.float32(v), fp8.E4M3)
    assert float(fp8.decode(c, fp8.E4M3)) == float(v), v
    return int(c)


def run_diag(rows_a, rows_b, K):
    """C = A B^T through fog_fp8_gemm (NT, scales 1); returns the diagonal as float64."""
    n = len(rows_a)
    A = np.zeros((n, K), np.uint8)
    B = np.zeros((n, K), np.uint8)
    for r, (ra, rb) in enumerate(zip(rows_a, rows_b)):
        for idx, v in ra.items():
            A[r, idx] = e4m3_of(v)
        for idx, v in rb.items():
            B[r, idx] = e4m3_of(v)
    C = torch.full((n, n), 0x7FC0, dtype=torch.int16, device="cuda")
    fog.fp8_gemm(fog.NT, n, n, K, dev(A), fog.E4M3, fscalar(1.0), dev(B), fog.E4M3, fscalar(1.0), C)
    torch.cuda.synchronize()
    Cf = (host_u16(C).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return np.diag(Cf), fp8.decode(A, fp8.E4M3), fp8.decode(B, fp8.E4M3)


def split_pow2(e):
    """Two E4M3-representable powers of two whose product is 2^e (each exponent within -6..8)."""
    ea = max(-6, min(8, e // 2))
    eb = e - ea
    assert -6 <= eb <= 8, e
    return 2.0 ** ea, 2.0 ** eb


@pytest.mark.parametrize("K", [64, 128])
def test_truncation_window_and_group_size(K):
    big_a, big_b = 256.0, 256.0                                  # |B| = 2^16
    cases = []                                                    # (kind, k, row of A, row of B, exact result)
    same = [(0, 1, 2), (0, 7, 3), (2, 5, 7), (8, 9, 15), (24, 31, 28), (56, 63, 60)]          # (+B, -B, small): one aligned group
    other = [(0, 1, 8), (6, 7, 8), (8, 15, 7), (0, 7, 63), (16, 17, 40), (56, 57, 55)]         # small outside the group(s) of +-B
    split = [(7, 8, 0), (7, 8, 15)]                                                            # +B and -B in neighbouring groups, small beside one of them
    for k in range(6, 23):
        sa, sb = split_pow2(16 - k)
        for sign in (1.0, -1.0):
            for (ip, im, js) in same:
                cases.append(("same", k, {ip: big_a, im: -big_a, js: sign * sa}, {ip: big_b, im: big_b, js: sb}, sign * sa * sb))
            for (ip, im, js) in other:
                cases.append(("other", k, {ip: big_a, im: -big_a, js: sign * sa}, {ip: big_b, im: big_b, js: sb}, sign * sa * sb))
            for (ip, im, js) in split:
                cases.append(("split", k, {ip: big_a, im: -big_a, js: sign * sa}, {ip: big_b, im: big_b, js: sb}, sign * sa * sb))
    # few-bit small products (1.75 x 1.75 = 49 / 16: six significant bits), same group: partially truncated
    for k in range(6, 20):
        sa, sb = split_pow2(16 - k)
        if sa * 1.75 <= 448 and sb * 1.75 <= 448:
            for (ip, im, js) in same[:3]:
                cases.append(("bits", k, {ip: big_a, im: -big_a, js: 1.75 * sa}, {ip: big_b, im: big_b, js: 1.75 * sb}, 3.0625 * sa * sb))
    got, Adec, Bdec = run_diag([c[2] for c in cases], [c[3] for c in cases], K)
    keep = mfma_model.MFMA_KEEP_BITS
    lost_same = {}
    for i, (kind, k, _, _, exact) in enumerate(cases):
        bound = mfma_model.dot_uncertainty(Adec[i:i + 1], Bdec[i:i + 1])[0, 0]
        err = abs(got[i] - exact)
        assert err <= bound, (kind, k, got[i], exact, bound)                      # (3), and the model's bound in every case
        if kind == "other":
            assert got[i] == exact, (kind, k, got[i], exact)                       # (2)
        if kind == "same" and k <= keep:
            assert got[i] == exact, (kind, k, got[i], exact)                       # (1)
        if kind == "same":
            lost_same.setdefault(k, []).append(got[i] == 0.0)
    for k in range(16, 23):
        assert all(lost_same[k]), k                                                # (4)
    first_loss = min(k for k, v in lost_same.items() if not all(not x for x in v))
    assert first_loss > keep
    print("small product first lost at 2^-%d of its group's largest (model keeps %d places)" % (first_loss, keep))

"""Pins for the oracle's scaled FP8 GEMM (CPU only)."""
import numpy as np
import pytest
import torch

from oracle import bf16, fp8, gemm, scaling
from paper_2505_20524_amd import synth

ONE = {fp8.E4M3: 0x38, fp8.E5M2: 0x3C}


def rand_codes(rng, shape, fmt):
    c = rng.integers(0, 256, size=shape, dtype=np.uint8)
    bad = ~np.isfinite(fp8.decode(c, fmt))
    c[bad] = 0
    return c


def operands(layout, A_mk, B_nk):
    """Lay out logical A[M,K], B[N,K] for the given layout."""
    if layout == gemm.NT:
        return A_mk, B_nk
    if layout == gemm.NN:
        return A_mk, np.ascontiguousarray(B_nk.T)
    return np.ascontiguousarray(A_mk.T), np.ascontiguousarray(B_nk.T)


@pytest.mark.parametrize("layout", [gemm.NT, gemm.NN, gemm.TN])
def test_identity_and_one_hot(layout):
    rng = np.random.default_rng(2)
    M, K = 9, 16
    A = rand_codes(rng, (M, K), fp8.E4M3)
    eye = np.where(np.eye(K, dtype=bool), ONE[fp8.E5M2], 0).astype(np.uint8)       # B = I in E5M2
    a, b = operands(layout, A, eye)
    C = gemm.fp8_gemm(layout, a, fp8.E4M3, 0.5, b, fp8.E5M2, 4.0)
    assert np.array_equal(C, 2.0 * fp8.decode(A, fp8.E4M3))
    # a permutation matrix moves columns
    perm = rng.permutation(K)
    Pm = np.zeros((K, K), np.uint8)
    Pm[np.arange(K), perm] = ONE[fp8.E4M3]                                         # B[n, perm[n]] = 1
    a, b = operands(layout, A, Pm)
    C = gemm.fp8_gemm(layout, a, fp8.E4M3, 1.0, b, fp8.E4M3, 1.0)
    assert np.array_equal(C, fp8.decode(A, fp8.E4M3)[:, perm])
    # one-hot A and one-hot B: a single non-zero at a known place (this catches a transposed operand)
    A1 = np.zeros((5, 7), np.uint8); A1[3, 2] = 0x40                                # 2.0 at (m=3,k=2)
    B1 = np.zeros((6, 7), np.uint8); B1[4, 2] = 0x44                                # 3.0 at (n=4,k=2)
    a, b = operands(layout, A1, B1)
    C = gemm.fp8_gemm(layout, a, fp8.E4M3, 1.0, b, fp8.E4M3, 1.0)
    want = np.zeros((5, 6)); want[3, 4] = 6.0
    assert np.array_equal(C, want)


@pytest.mark.parametrize("layout", [gemm.NT, gemm.NN, gemm.TN])
def test_small_integers_equal_integer_matmul(layout):
    """Integer data with power-of-two scales: the FP8 route of Appendix E is exact."""
    rng = np.random.default_rng(3)
    M, N, K = 23, 17, 64
    Ai = rng.integers(-8, 9, size=(M, K))
    Bi = rng.integers(-4, 5, size=(N, K))
    rho_a, rho_b = np.float32(4.0), np.float32(8.0)
    Ab = synth.f32_to_bf16_bits((Ai / 4.0).astype(np.float32))
    Bb = synth.f32_to_bf16_bits((Bi / 8.0).astype(np.float32))
    A8 = scaling.quantize(Ab, rho_a, fp8.E4M3)
    B8 = scaling.quantize(Bb, rho_b, fp8.E5M2)
    a, b = operands(layout, A8, B8)
    C = gemm.fp8_gemm(layout, a, fp8.E4M3, np.float32(0.25), b, fp8.E5M2, np.float32(0.125))
    assert np.array_equal(C, (Ai @ Bi.T).astype(np.float64) / 32.0)


@pytest.mark.parametrize("layout", [gemm.NT, gemm.NN, gemm.TN])
def test_against_library_matmul_and_rows(layout):
    rng = np.random.default_rng(4)
    M, N, K = 33, 29, 96
    A = rand_codes(rng, (M, K), fp8.E4M3)
    B = rand_codes(rng, (N, K), fp8.E5M2)
    At = torch.from_numpy(A.copy()).view(torch.float8_e4m3fn).to(torch.float64)
    Bt = torch.from_numpy(B.copy()).view(torch.float8_e5m2).to(torch.float64)
    sa, sb = np.float32(0.37), np.float32(1.9e-3)
    lib = (float(sa) * float(sb)) * (At @ Bt.T).numpy()
    a, b = operands(layout, A, B)
    C = gemm.fp8_gemm(layout, a, fp8.E4M3, sa, b, fp8.E5M2, sb)
    assert np.allclose(C, lib, rtol=1e-13, atol=1e-13 * np.abs(lib).max())
    rows = [0, 5, 32]
    Cr = gemm.fp8_gemm_rows(layout, a, fp8.E4M3, sa, b, fp8.E5M2, sb, rows)
    assert np.array_equal(Cr, C[rows])
    assert np.array_equal(gemm.to_bf16(C), bf16.f64_round(C))


def test_end_to_end_matches_unquantised_product_within_fp8_error():
    """GEMM(X, Y) of Appendix E approximates X Y^T; the error is what per-tensor E4M3 allows."""
    x, w, _ = synth.small_linear(5, 64, 48, 256, outlier_cols=0)
    ax, aw = scaling.amax(x), scaling.amax(w)
    rx, rxi = scaling.compute_scale(ax, fp8.E4M3)
    rw, rwi = scaling.compute_scale(aw, fp8.E4M3)
    C = gemm.fp8_gemm(gemm.NT, scaling.quantize(x, rx, fp8.E4M3), fp8.E4M3, rxi,
                      scaling.quantize(w, rw, fp8.E4M3), fp8.E4M3, rwi)
    ref = bf16.bits_to_f64(x) @ bf16.bits_to_f64(w).T
    rel = np.linalg.norm(C - ref) / np.linalg.norm(ref)
    assert 1e-3 < rel < 6e-2        # ~2^-4/sqrt(3) per operand; not zero, not broken

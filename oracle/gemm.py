"""End-to-end FP8 matrix product (Appendix E):

    GEMM(X, Y) = 1 / (rho(X) rho(Y)) * FP8GEMM(FP8cast(rho(X) X), FP8cast(rho(Y) Y))

The operands arrive already cast (uint8 codes) together with the reciprocal
scales.  The product of the decoded operands is accumulated in float64 and
multiplied by the two reciprocal scales; the result is kept in float64
(`to_bf16` states it in the output format the paper gives FP8GEMM).

Layouts (row-major), covering forward, data-gradient and weight-gradient
products of a linear layer Y = X W^T (Appendix E, table of FP8 methods: the
linear operators run in FP8 in both passes):
    NT: C[M,N] = A[M,K] . B[N,K]^T
    NN: C[M,N] = A[M,K] . B[K,N]
    TN: C[M,N] = A[K,M]^T . B[K,N]
"""
import numpy as np

from . import bf16, fp8

NT, NN, TN = 0, 1, 2


def fp8_gemm(layout, A, fmt_a, sinv_a, B, fmt_b, sinv_b):
    a = fp8.decode(A, fmt_a)
    b = fp8.decode(B, fmt_b)
    if layout == NT:
        acc = a @ b.T
    elif layout == NN:
        acc = a @ b
    elif layout == TN:
        acc = a.T @ b
    else:
        raise ValueError("layout")
    return np.float64(sinv_a) * np.float64(sinv_b) * acc


def fp8_gemm_rows(layout, A, fmt_a, sinv_a, B, fmt_b, sinv_b, rows):
    """Selected output rows only (same arithmetic), for sizes too large to compute whole."""
    rows = np.asarray(rows)
    a = fp8.decode(A, fmt_a)
    b = fp8.decode(B, fmt_b)
    if layout == NT:
        acc = a[rows] @ b.T
    elif layout == NN:
        acc = a[rows] @ b
    elif layout == TN:
        acc = a[:, rows].T @ b
    else:
        raise ValueError("layout")
    return np.float64(sinv_a) * np.float64(sinv_b) * acc


def to_bf16(c):
    return bf16.f64_round(c)

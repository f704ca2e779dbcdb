"""GPU parity: scaled FP8 GEMM (NT / NN / TN) against the float64 oracle."""
import numpy as np
import pytest
import torch

from oracle import fp8, gemm, scaling
from paper_2505_20524_amd import fog, synth
from parity import check_bf16, check_gemm_elementwise, dev, fscalar, host_u16

pytestmark = pytest.mark.gpu


def lay(layout, A_mk, B_nk):
    if layout == gemm.NT:
        return A_mk, B_nk
    if layout == gemm.NN:
        return A_mk, np.ascontiguousarray(B_nk.T)
    return np.ascontiguousarray(A_mk.T), np.ascontiguousarray(B_nk.T)


def run_gemm(layout, A8, fa, sa, B8, fb, sb, M, N, K, ldc_pad=0):
    C = torch.full((M, N + ldc_pad), 0x7FC0, dtype=torch.int16, device="cuda")[:, :N] if ldc_pad else \
        torch.full((M, N), 0x7FC0, dtype=torch.int16, device="cuda")
    fog.fp8_gemm(layout, M, N, K, dev(A8), fa, fscalar(sa), dev(B8), fb, fscalar(sb), C)
    torch.cuda.synchronize()
    return host_u16(C)


def absdot(layout, a, fa, sa, b, fb, sb):
    """sinv_a sinv_b (|decode(A)| x |decode(B)|): the magnitude each output element accumulates."""
    A, B = np.abs(fp8.decode(a, fa)), np.abs(fp8.decode(b, fb))
    acc = A @ B.T if layout == gemm.NT else (A @ B if layout == gemm.NN else A.T @ B)
    return np.float64(sa) * np.float64(sb) * acc


def quantized_layer(seed, M, N, K, fa=fp8.E4M3, fb=fp8.E4M3):
    x, w, _ = synth.small_linear(seed, M, N, K)
    rx, rxi = scaling.compute_scale(scaling.amax(x), fa)
    rw, rwi = scaling.compute_scale(scaling.amax(w), fb)
    return scaling.quantize(x, rx, fa), rxi, scaling.quantize(w, rw, fb), rwi


SHAPES = [(512, 1024, 1024), (304, 528, 384), (272, 16, 144), (16, 272, 16), (1024, 512, 2048), (48, 48, 4096)]


@pytest.mark.parametrize("layout", [gemm.NT, gemm.NN, gemm.TN])
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_parity(layout, M, N, K):
    A8, sa, B8, sb = quantized_layer(M + N + K, M, N, K)
    a, b = lay(layout, A8, B8)
    ref = gemm.fp8_gemm(layout, a, fp8.E4M3, sa, b, fp8.E4M3, sb)
    got = run_gemm(layout, a, fp8.E4M3, sa, b, fp8.E4M3, sb, M, N, K)
    stats = check_bf16(got, ref, what="gemm %d %dx%dx%d" % (layout, M, N, K))
    assert stats["max_steps"] <= 1
    # the tensor-normalised gate says little about elements far below the maximum (the x50 outlier channels make most
    # of them so): each element against its own value and its own accumulated magnitude
    check_gemm_elementwise(got, ref, absdot(layout, a, fp8.E4M3, sa, b, fp8.E4M3, sb), what="gemm %d %dx%dx%d" % (layout, M, N, K))


@pytest.mark.parametrize("layout", [gemm.NT, gemm.NN, gemm.TN])
def test_gemm_padded_leading_dimensions(layout):
    """Operands and result as views of wider buffers (lda, ldb, ldc larger than the rows): nothing outside the
    views is read into the result or written."""
    M, N, K = 304, 528, 400
    A8, sa, B8, sb = quantized_layer(77, M, N, K)
    a, b = lay(layout, A8, B8)
    ref = gemm.fp8_gemm(layout, a, fp8.E4M3, sa, b, fp8.E4M3, sb)
    pa, pb, pc = 16, 48, 8
    abuf = torch.full((a.shape[0], a.shape[1] + pa), 0x7E, dtype=torch.uint8, device="cuda")     # padding = largest code: a leak would show
    bbuf = torch.full((b.shape[0], b.shape[1] + pb), 0x7E, dtype=torch.uint8, device="cuda")
    abuf[:, :a.shape[1]] = dev(a)
    bbuf[:, :b.shape[1]] = dev(b)
    cbuf = torch.full((M, N + pc), 0x7FC0, dtype=torch.int16, device="cuda")
    fog.fp8_gemm(layout, M, N, K, abuf[:, :a.shape[1]], fp8.E4M3, fscalar(sa), bbuf[:, :b.shape[1]], fp8.E4M3, fscalar(sb), cbuf[:, :N])
    torch.cuda.synchronize()
    assert (cbuf[:, N:] == 0x7FC0).all()
    check_bf16(host_u16(cbuf[:, :N].contiguous()), ref, what="padded ld, layout %d" % layout)


def test_gemm_ragged_rows_nt():
    """NT takes any M and N (rows of the operands); K only has to be a multiple of 16."""
    for (M, N, K) in [(1, 1, 16), (257, 259, 160), (300, 37, 128), (5, 700, 400)]:
        A8, sa, B8, sb = quantized_layer(M * 7 + N, M, N, K)
        ref = gemm.fp8_gemm(gemm.NT, A8, fp8.E4M3, sa, B8, fp8.E4M3, sb)
        got = run_gemm(gemm.NT, A8, fp8.E4M3, sa, B8, fp8.E4M3, sb, M, N, K, ldc_pad=(3 if N % 2 else 0))
        check_bf16(got, ref, what="ragged %dx%dx%d" % (M, N, K))


@pytest.mark.parametrize("layout", [gemm.NT, gemm.NN, gemm.TN])
@pytest.mark.parametrize("fa,fb", [(fp8.E5M2, fp8.E4M3), (fp8.E4M3, fp8.E5M2), (fp8.E5M2, fp8.E5M2)])
def test_gemm_mixed_formats(layout, fa, fb):
    M, N, K = 320, 288, 256
    A8, sa, B8, sb = quantized_layer(17, M, N, K, fa, fb)
    a, b = lay(layout, A8, B8)
    ref = gemm.fp8_gemm(layout, a, fa, sa, b, fb, sb)
    got = run_gemm(layout, a, fa, sa, b, fb, sb, M, N, K)
    check_bf16(got, ref, what="formats")
    check_gemm_elementwise(got, ref, absdot(layout, a, fa, sa, b, fb, sb), what="formats")


@pytest.mark.parametrize("layout", [gemm.NT, gemm.NN, gemm.TN])
def test_gemm_exact_cases(layout):
    """Small integers with power-of-two scales: the result is exact and bf16-representable."""
    rng = np.random.default_rng(5)
    M, N, K = 288, 272, 256
    Ai = rng.integers(-2, 3, size=(M, K)); Bi = rng.integers(-2, 3, size=(N, K))
    Ai[rng.random((M, K)) < 0.7] = 0; Bi[rng.random((N, K)) < 0.7] = 0      # keep |sums| < 256: exact in bf16
    A8 = scaling.quantize(synth.f32_to_bf16_bits(Ai.astype(np.float32)), np.float32(1), fp8.E4M3)
    B8 = scaling.quantize(synth.f32_to_bf16_bits(Bi.astype(np.float32)), np.float32(1), fp8.E5M2)
    a, b = lay(layout, A8, B8)
    got = run_gemm(layout, a, fp8.E4M3, 0.5, b, fp8.E5M2, 0.25, M, N, K)
    want = (Ai @ Bi.T) / 8.0
    assert np.abs(Ai @ Bi.T).max() < 256
    assert np.array_equal(synth.bf16_bits_to_f32(got).astype(np.float64), want)
    # one-hot operands: a single non-zero at a known place
    A1 = np.zeros((M, K), np.uint8); B1 = np.zeros((N, K), np.uint8)
    A1[200, 77] = 0x40; B1[131, 77] = 0x44
    a, b = lay(layout, A1, B1)
    got = synth.bf16_bits_to_f32(run_gemm(layout, a, fp8.E4M3, 1.0, b, fp8.E4M3, 1.0, M, N, K))
    want = np.zeros((M, N), np.float32); want[200, 131] = 6.0
    assert np.array_equal(got, want)


def test_gemm_k_zero_and_empty():
    C = torch.full((32, 48), 0x7FC0, dtype=torch.int16, device="cuda")
    one = fscalar(1.0)
    lib = fog.load()
    st = torch.cuda.current_stream().cuda_stream
    assert lib.fog_fp8_gemm(0, 32, 48, 0, None, 0, 0, one.data_ptr(), None, 0, 0, one.data_ptr(), C.data_ptr(), 48, None, 0, st) == 0
    torch.cuda.synchronize()
    assert (C.cpu().numpy() == 0).all()
    assert lib.fog_fp8_gemm(0, 0, 48, 16, None, 0, 16, one.data_ptr(), None, 0, 16, one.data_ptr(), C.data_ptr(), 48, None, 0, st) == 0


def test_gemm_argument_errors():
    lib = fog.load()
    st = torch.cuda.current_stream().cuda_stream
    A = torch.zeros(64 * 64, dtype=torch.uint8, device="cuda")
    C = torch.zeros(64 * 64, dtype=torch.int16, device="cuda")
    one = fscalar(1.0)
    p, o = A.data_ptr(), one.data_ptr()
    assert lib.fog_fp8_gemm(0, 64, 64, 64, None, 0, 64, o, p, 0, 64, o, C.data_ptr(), 64, None, 0, st) == 1
    assert lib.fog_fp8_gemm(0, 64, 64, 64, p, 0, 32, o, p, 0, 64, o, C.data_ptr(), 64, None, 0, st) == 2
    assert lib.fog_fp8_gemm(0, 64, 64, 64, p + 1, 0, 64, o, p, 0, 64, o, C.data_ptr(), 64, None, 0, st) == 3
    assert lib.fog_fp8_gemm(0, 64, 64, 40, p, 0, 48, o, p, 0, 48, o, C.data_ptr(), 64, None, 0, st) == 4
    assert lib.fog_fp8_gemm(1, 64, 40, 64, p, 0, 64, o, p, 0, 48, o, C.data_ptr(), 64, None, 0, st) == 4
    assert lib.fog_fp8_gemm(5, 64, 64, 64, p, 0, 64, o, p, 0, 64, o, C.data_ptr(), 64, None, 0, st) == 4
    assert lib.fog_fp8_gemm(0, -1, 64, 64, p, 0, 64, o, p, 0, 64, o, C.data_ptr(), 64, None, 0, st) == 2


def test_config2_full_size_all_three_products():
    """Config 2 whole (tokens 4096, in 2048, out 8192): forward, data gradient, weight gradient,
    each both in its native layout and as NT on the transposed copies the cast kernel emits."""
    cfg = synth.CONFIGS[2]
    t = synth.linear_tensors(cfg, 0)
    M, N, K = 4096, 8192, 2048
    dv = {}
    ora = {}
    for name, fmt in (("X", fp8.E4M3), ("W", fp8.E4M3), ("dY", fp8.E5M2)):
        xb = t[name]
        xd = dev(xb)
        am, s, si = (torch.zeros(1, device="cuda") for _ in range(3))
        fog.amax(xd, am); fog.scale(am, fmt, s, si)
        q = torch.zeros(xb.shape, dtype=torch.uint8, device="cuda")
        qT = torch.zeros(xb.shape[::-1], dtype=torch.uint8, device="cuda")
        fog.quantize(xd, fmt, s, q=q, qT=qT)
        rho, rinv = scaling.compute_scale(scaling.amax(xb), fmt)
        want = scaling.quantize(xb, rho, fmt)
        assert np.float32(si.item()) == rinv
        assert np.array_equal(q.cpu().numpy(), want) and np.array_equal(qT.cpu().numpy(), want.T)
        dv[name] = (q, qT, si)
        ora[name] = (want, rinv)

    def gpu(layout, m, n, k, A, fa, sa, B, fb, sb):
        C = torch.zeros((m, n), dtype=torch.int16, device="cuda")
        fog.fp8_gemm(layout, m, n, k, A, fa, sa, B, fb, sb, C)
        torch.cuda.synchronize()
        return host_u16(C)

    X, W, dY = ora["X"], ora["W"], ora["dY"]
    ref = gemm.fp8_gemm(gemm.NT, X[0], fp8.E4M3, X[1], W[0], fp8.E4M3, W[1])                     # Y = X W^T
    check_bf16(gpu(fog.NT, M, N, K, dv["X"][0], 0, dv["X"][2], dv["W"][0], 0, dv["W"][2]), ref, what="fwd")
    ref = gemm.fp8_gemm(gemm.NN, dY[0], fp8.E5M2, dY[1], W[0], fp8.E4M3, W[1])                   # dX = dY W
    check_bf16(gpu(fog.NN, M, K, N, dv["dY"][0], 1, dv["dY"][2], dv["W"][0], 0, dv["W"][2]), ref, what="dgrad NN")
    check_bf16(gpu(fog.NT, M, K, N, dv["dY"][0], 1, dv["dY"][2], dv["W"][1], 0, dv["W"][2]), ref, what="dgrad NT(W^T)")
    ref = gemm.fp8_gemm(gemm.TN, dY[0], fp8.E5M2, dY[1], X[0], fp8.E4M3, X[1])                   # dW = dY^T X
    check_bf16(gpu(fog.TN, N, K, M, dv["dY"][0], 1, dv["dY"][2], dv["X"][0], 0, dv["X"][2]), ref, what="wgrad TN")
    check_bf16(gpu(fog.NT, N, K, M, dv["dY"][1], 1, dv["dY"][2], dv["X"][1], 0, dv["X"][2]), ref, what="wgrad NT(dY^T, X^T)")


def run_gemm_ws(layout, a, fa, sa, b, fb, sb, M, N, K, ws_bytes=None):
    """fog_fp8_gemm with the workspace the query asks for (or `ws_bytes`); returns (C bits, bytes the query asked for)."""
    need = fog.fp8_gemm_workspace(layout, M, N, K)
    n = need if ws_bytes is None else ws_bytes
    ws = torch.full((max(n, 16),), 0xFF, dtype=torch.uint8, device="cuda") if n else None      # NaN patterns: a partial read before written would show
    C = torch.full((M, N), 0x7FC0, dtype=torch.int16, device="cuda")
    fog.fp8_gemm(layout, M, N, K, dev(a), fa, fscalar(sa), dev(b), fb, fscalar(sb), C, workspace=ws)
    torch.cuda.synchronize()
    return host_u16(C), need


SPLIT_SHAPES = [   # few output tiles, long contraction: the launches the split is for
    (gemm.TN, 2048, 2048, 16384),     # config 4: weight gradient of the output projection (64 tiles)
    (gemm.NN, 4096, 2048, 8192),      # config 2: data gradient (128 tiles)
    (gemm.NT, 256, 256, 32768),       # one tile
    (gemm.NN, 1024, 1024, 8192),      # 16 tiles
    (gemm.NT, 300, 200, 5008),        # ragged edges, contraction not a multiple of the chunk or of a K-step
    (gemm.TN, 272, 528, 4112),        # K-major operands with a ragged contraction
    (gemm.NN, 48, 1040, 12304),
]


@pytest.mark.parametrize("layout,M,N,K", SPLIT_SHAPES)
def test_gemm_contraction_split(layout, M, N, K):
    """With the workspace the query asks for, launches of few tiles are cut along the contraction (binary32 partial
    tiles, reduced in a fixed order): same gate as the unsplit kernel, the same bits on a second call, and without a
    workspace (or with one that is too small) the unsplit kernel answers inside the same gate."""
    fa, fb = (fp8.E5M2, fp8.E4M3) if layout != gemm.NT else (fp8.E4M3, fp8.E4M3)
    A8, sa, B8, sb = quantized_layer(M + 3 * N + K, M, N, K, fa, fb)
    a, b = lay(layout, A8, B8)
    ref = gemm.fp8_gemm(layout, a, fa, sa, b, fb, sb)
    got, need = run_gemm_ws(layout, a, fa, sa, b, fb, sb, M, N, K)
    assert need > 0 and need % (256 * 256 * 4) == 0, "the query did not ask for a split on this shape"
    st = check_bf16(got, ref, what="split %d %dx%dx%d" % (layout, M, N, K))
    assert st["max_steps"] <= 1
    check_gemm_elementwise(got, ref, absdot(layout, a, fa, sa, b, fb, sb), what="split %d %dx%dx%d" % (layout, M, N, K))
    again, _ = run_gemm_ws(layout, a, fa, sa, b, fb, sb, M, N, K)
    assert np.array_equal(got, again)                      # deterministic: no atomics, fixed order of the chunks
    for small in (0, need - 1):
        unsplit, _ = run_gemm_ws(layout, a, fa, sa, b, fb, sb, M, N, K, ws_bytes=small)
        check_bf16(unsplit, ref, what="unsplit fallback")
    # the two routes differ only in the order of binary32 additions: at most one bf16 step, on few elements
    steps = np.abs(got.astype(np.int32) - unsplit.astype(np.int32))
    assert steps.max() <= 1 and (steps > 0).mean() < 0.05


def test_gemm_split_exact_integers_and_query():
    """Small integers: every partial sum is exact, so split and unsplit give identical, exact results; shapes with
    enough tiles ask for no workspace."""
    rng = np.random.default_rng(11)
    M, N, K = 256, 512, 16384
    Ai = rng.integers(-2, 3, size=(M, K)); Bi = rng.integers(-2, 3, size=(N, K))
    Ai[rng.random((M, K)) < 0.97] = 0; Bi[rng.random((N, K)) < 0.9] = 0
    assert np.abs(Ai @ Bi.T).max() < 256
    A8 = scaling.quantize(synth.f32_to_bf16_bits(Ai.astype(np.float32)), np.float32(1), fp8.E4M3)
    B8 = scaling.quantize(synth.f32_to_bf16_bits(Bi.astype(np.float32)), np.float32(1), fp8.E4M3)
    got, need = run_gemm_ws(gemm.NT, A8, fp8.E4M3, 0.5, B8, fp8.E4M3, 0.5, M, N, K)
    assert need > 0
    assert np.array_equal(synth.bf16_bits_to_f32(got).astype(np.float64), (Ai @ Bi.T) / 4.0)
    for (layout, m, n, k) in [(gemm.NT, 8192, 12288, 4096), (gemm.TN, 14336, 4096, 8192), (gemm.NT, 512, 1024, 1024)]:
        assert fog.fp8_gemm_workspace(layout, m, n, k) == 0

"""GPU: the benchmark's measurement helper (include/fog_probe.h) runs, reports rates that are physically possible and
rejects bad arguments.  It is not part of the hot path; this only keeps the benchmark's --ceilings leg honest."""
import ctypes

import pytest
import torch

from paper_2505_20524_amd import fog

pytestmark = pytest.mark.gpu


def test_mfma_rate_probe_reports_a_possible_rate_and_checks_arguments():
    pat = torch.full((65536,), 0x38, dtype=torch.uint8, device="cuda")
    sink = torch.empty(1024 * 256, device="cuda")
    tf, ghz = fog.probe_mfma_rate(pat, 2000, sink)
    assert 500.0 < tf < 5033.0 * 1.05          # below the published dense-FP8 peak (small margin for clock tolerance), far above a stall
    assert 0.3 < ghz < 2.6
    lib = fog.load()
    st = torch.cuda.current_stream().cuda_stream
    a, b = ctypes.c_double(0), ctypes.c_double(0)
    call = lambda p, it, s, sb: lib.fog_probe_mfma_rate(p, it, s, sb, ctypes.byref(a), ctypes.byref(b), st)
    assert call(None, 10, sink.data_ptr(), sink.numel() * 4) == 1
    assert call(pat.data_ptr(), 0, sink.data_ptr(), sink.numel() * 4) == 2
    assert call(pat.data_ptr() + 1, 10, sink.data_ptr(), sink.numel() * 4) == 3
    assert call(pat.data_ptr(), 10, sink.data_ptr(), 64) == 5


def test_attention_loop_probe_orders_its_three_timings():
    sink = torch.empty(1024 * 256, device="cuda")
    t_all, t_mfma, t_valu = (fog.probe_attention_loop(w, 2, 500, sink) for w in (0, 1, 2))
    assert 0 < t_mfma <= t_all * 1.05 and 0 < t_valu <= t_all * 1.05        # a part cannot take longer than the whole
    assert t_all <= (t_mfma + t_valu) * 1.15                                 # and the whole no longer than the parts in sequence
    t_ilv = fog.probe_attention_loop(3, 2, 500, sink)                        # the same work, interleaved inside the wave
    assert t_mfma <= t_ilv * 1.05 and t_ilv <= (t_mfma + t_valu) * 1.15
    lib = fog.load()
    ns = ctypes.c_double(0)
    st = torch.cuda.current_stream().cuda_stream
    assert lib.fog_probe_attention_loop(0, 4, 10, sink.data_ptr(), sink.numel() * 4, ctypes.byref(ns), st) == 2
    assert lib.fog_probe_attention_loop(4, 1, 10, sink.data_ptr(), sink.numel() * 4, ctypes.byref(ns), st) == 2
    assert lib.fog_probe_attention_loop(0, 1, 10, None, 0, ctypes.byref(ns), st) == 1
    assert lib.fog_probe_attention_loop(0, 2, 10, sink.data_ptr(), 64, ctypes.byref(ns), st) == 5


def test_coissue_probe_shows_the_matrix_instruction_and_checks_arguments():
    sink = torch.empty(1024 * 256 + 4096, device="cuda")
    alone = fog.probe_mfma_coissue(0, 0, True, 500, sink)
    assert 60.0 < alone < 80.0                       # 16 passes of 4 cycles, back to back
    few = fog.probe_mfma_coissue(0, 4, True, 500, sink)
    many = fog.probe_mfma_coissue(0, 32, True, 500, sink)
    bare = fog.probe_mfma_coissue(0, 32, False, 500, sink)
    assert few < alone * 1.15                        # a few vector operations hide under the matrix instruction
    assert bare < many < bare + 64.0                 # and many of them hide most of the matrix instruction in turn
    lib = fog.load()
    cyc = ctypes.c_double(0)
    st = torch.cuda.current_stream().cuda_stream
    call = lambda op, n, p, sb: lib.fog_probe_mfma_coissue(op, n, 1, 10, p, sb, ctypes.byref(cyc), st)
    assert call(4, 4, sink.data_ptr(), sink.numel() * 4) == 2
    assert call(0, 5, sink.data_ptr(), sink.numel() * 4) == 2
    assert call(0, 4, None, 0) == 1
    assert call(0, 4, sink.data_ptr() + 4, sink.numel() * 4 - 4) == 3
    assert call(0, 4, sink.data_ptr(), 64) == 5


def test_products_only_gemm_probe_runs_writes_nothing_and_checks_arguments():
    M, N, K = 512, 768, 1024
    g = torch.Generator(device="cuda"); g.manual_seed(3)
    A = torch.randint(0, 0x78, (M, K), dtype=torch.uint8, device="cuda", generator=g)
    B = torch.randint(0, 0x78, (N, K), dtype=torch.uint8, device="cuda", generator=g)
    one = torch.ones(1, device="cuda")
    C = torch.full((M, N), 0x1234, dtype=torch.int16, device="cuda")
    fog.probe_gemm_products_only(M, N, K, A, one, B, one, C)
    torch.cuda.synchronize()
    assert bool((C == 0x1234).all())                  # no tile has an epilogue: C is untouched
    lib = fog.load()
    st = torch.cuda.current_stream().cuda_stream
    call = lambda m, n, k, a, c: lib.fog_probe_gemm_products_only(m, n, k, a, K, B.data_ptr(), K, one.data_ptr(), one.data_ptr(), c, N, st)
    assert call(M + 1, N, K, A.data_ptr(), C.data_ptr()) == 4
    assert call(M, N, K, None, C.data_ptr()) == 1
    assert call(M, N, K, A.data_ptr() + 1, C.data_ptr()) == 3
    assert call(0, N, K, A.data_ptr(), C.data_ptr()) == 2


def test_cross_wave_probe_shows_overlap_between_waves_and_checks_arguments():
    """A matrix-only wave keeps its 64 cycles per instruction while a vector-only wave shares its SIMD, and the vector wave
    slows down by far less than the matrix time it runs under (the two units do overlap across waves)."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.zeros(cus * 512 + cus * 4 + 16, device="cuda")
    _, v_alone = fog.probe_mfma_cross_wave(0, 8, 0, 500, sink)
    m_alone, _ = fog.probe_mfma_cross_wave(0, 8, 500, 0, sink)
    m_long, v_under = fog.probe_mfma_cross_wave(0, 8, 1500, 500, sink)      # 1500 x 512 cycles of matrix work outlast the vector trips
    assert 63.0 <= m_alone <= 70.0 and 63.0 <= m_long <= 70.0
    assert 30.0 <= v_alone <= 60.0                                            # eight fused multiply-adds: 4-5 cycles each plus the loop
    assert v_alone <= v_under <= v_alone + 0.5 * 64.0
    lib = fog.load()
    import ctypes as C
    a, b = C.c_double(0.0), C.c_double(0.0)
    nbytes = sink.numel() * 4
    call = lib.fog_probe_mfma_cross_wave
    assert call(0, 8, 10, 10, sink.data_ptr(), nbytes, None, C.byref(b), None) == 1
    assert call(4, 8, 10, 10, sink.data_ptr(), nbytes, C.byref(a), C.byref(b), None) == 2
    assert call(0, 16, 10, 10, sink.data_ptr(), nbytes, C.byref(a), C.byref(b), None) == 2
    assert call(0, 8, 0, 0, sink.data_ptr(), nbytes, C.byref(a), C.byref(b), None) == 2
    assert call(0, 8, 10, 10, sink.data_ptr() + 4, nbytes - 4, C.byref(a), C.byref(b), None) == 3
    assert call(0, 8, 10, 10, sink.data_ptr(), 1024, C.byref(a), C.byref(b), None) == 5

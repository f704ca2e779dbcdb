"""GPU parity: abs-max, scale and cast kernels against the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

from oracle import fp8, scaling
from paper_2505_20524_amd import fog, synth
from parity import dev, fscalar

pytestmark = pytest.mark.gpu


def gpu_amax(xb):
    out = torch.full((1,), -1.0, device="cuda")
    fog.amax(dev(xb), out)
    return np.float32(out.item())


@pytest.mark.parametrize("n", [0, 1, 7, 8, 9, 1023, 4096, 100003, 512 * 1024, 4096 * 2048 + 5])
def test_amax_bit_exact(n):
    rng = np.random.default_rng(n)
    xb = synth.f32_to_bf16_bits(rng.standard_normal(n).astype(np.float32) * 3)
    if n:
        assert gpu_amax(xb) == scaling.amax(xb)
        for pos in {0, n - 1, n // 2, max(n - 3, 0)}:
            y = xb.copy(); y[pos] = 0xC2C8            # plant -100 at an edge position
            assert gpu_amax(y) == np.float32(100.0)
    else:
        out = torch.full((1,), -1.0, device="cuda")
        fog.load().fog_amax(None, 0, out.data_ptr(), torch.cuda.current_stream().cuda_stream)
        assert out.item() == 0.0


@pytest.mark.parametrize("fmt", [fp8.E4M3, fp8.E5M2])
def test_scale_bit_exact(fmt):
    vals = [0.0, 1.0, 3.0, 448.0, 1e-3, 7.3e4, 1e-44, 3e38, np.inf, np.nan, 0.1234567, 100.0]
    for a in vals:
        for margin in (0, 1, -2):
            s, si = torch.zeros(1, device="cuda"), torch.zeros(1, device="cuda")
            fog.scale(fscalar(a), fmt, s, si, margin=margin)
            rho, rinv = scaling.compute_scale(np.float32(a), fmt, margin)
            assert np.float32(s.item()).tobytes() == rho.tobytes(), (a, margin)
            assert np.float32(si.item()).tobytes() == rinv.tobytes(), (a, margin)


def test_scale_delayed_history():
    L = 1024                                           # the paper's history length (Appendix E)
    rng = np.random.default_rng(0)
    hist = rng.uniform(0.1, 5.0, L).astype(np.float32)
    h = dev(hist)
    s, si = torch.zeros(1, device="cuda"), torch.zeros(1, device="cuda")
    ref = hist.copy()
    for step in range(5):
        na = np.float32(7.0 if step == 2 else 0.3)
        fog.scale_delayed(h, fscalar(na), fp8.E4M3, s, si)
        ref = scaling.history_update(ref, na)
        rho, rinv = scaling.history_scale(ref, fp8.E4M3)
        assert np.array_equal(h.cpu().numpy(), ref)
        assert np.float32(s.item()) == rho and np.float32(si.item()) == rinv
    for L2 in (1, 3, 255, 256, 257, 700):
        hist = rng.uniform(0.1, 5.0, L2).astype(np.float32)
        h = dev(hist)
        fog.scale_delayed(h, fscalar(9.5), fp8.E5M2, s, si)
        ref = scaling.history_update(hist, 9.5)
        assert np.array_equal(h.cpu().numpy(), ref)
        assert np.float32(s.item()) == scaling.history_scale(ref, fp8.E5M2)[0]


CASES = [  # rows, cols, ldx extra, transpose
    (512, 1024, 0, False), (512, 1024, 0, True), (4096, 2048, 0, True), (272, 400, 0, True),
    (272, 400, 16, True), (100, 48, 0, True), (33, 17, 0, True), (33, 17, 3, False), (1, 16, 0, False),
    (16, 16, 0, True), (129, 144, 0, False), (384, 8192, 32, True),
]


@pytest.mark.parametrize("fmt", [fp8.E4M3, fp8.E5M2])
@pytest.mark.parametrize("rows,cols,pad,tr", CASES)
def test_quantize_bit_exact(fmt, rows, cols, pad, tr):
    rng = np.random.default_rng(rows * 131 + cols)
    x = rng.standard_normal((rows, cols + pad)).astype(np.float32)
    x[:, : min(3, cols)] *= 60.0
    x[0, 0] = 0.0
    xb = synth.f32_to_bf16_bits(x)
    view = xb[:, :cols]
    a = scaling.amax(view)
    rho, _ = scaling.compute_scale(a, fmt)
    want = scaling.quantize(view, rho, fmt)
    xd = dev(xb)[:, :cols]
    q = torch.full((rows, cols + pad), 0x55, dtype=torch.uint8, device="cuda")[:, :cols]
    qT = torch.full((cols, rows + pad), 0x55, dtype=torch.uint8, device="cuda")[:, :rows] if tr else None
    am = torch.full((1,), -1.0, device="cuda")
    fog.quantize(xd, fmt, fscalar(rho), q=q, qT=qT, amax_out=am)
    assert np.array_equal(q.cpu().numpy(), want)
    if tr:
        assert np.array_equal(qT.cpu().numpy(), want.T)
        # transposed output alone
        qT2 = torch.zeros((cols, rows), dtype=torch.uint8, device="cuda")
        fog.quantize(xd, fmt, fscalar(rho), q=None, qT=qT2)
        assert np.array_equal(qT2.cpu().numpy(), want.T)
    assert np.float32(am.item()) == a
    # padding untouched
    if pad:
        full = q._base if q._base is not None else q
        assert (full.cpu().numpy()[:, cols:] == 0x55).all()


def test_quantize_all_bf16_values_and_saturation():
    """Every finite bf16 value through the kernel at several scales, incl. ones that overflow the format."""
    allb = np.arange(65536, dtype=np.uint16)
    fin = np.isfinite(synth.bf16_bits_to_f32(allb))
    xb = allb[fin]
    n = (xb.size // 16) * 16
    xb = xb[:n].reshape(-1, 16)
    xd = dev(xb)
    for fmt in (fp8.E4M3, fp8.E5M2):
        for rho in (1.0, 448.0 / 3.7, 1e-3, 3.1e4, 1e30, 1e-30):
            q = torch.zeros(xb.shape, dtype=torch.uint8, device="cuda")
            fog.quantize(xd, fmt, fscalar(rho), q=q)
            want = scaling.quantize(xb, np.float32(rho), fmt)
            assert np.array_equal(q.cpu().numpy(), want), (fmt, rho)


def test_jit_flow_config1_tensors():
    """amax -> scale -> cast on config-1 tensors (X with 4 outlier channels x50, W ~ N(0, 0.02))."""
    cfg = synth.CONFIGS[1]
    t = synth.linear_tensors(cfg, 0, want=("X", "W"))
    for name in ("X", "W"):
        xb = t[name]
        xd = dev(xb)
        am, s, si = (torch.zeros(1, device="cuda") for _ in range(3))
        fog.amax(xd, am)
        fog.scale(am, fp8.E4M3, s, si)
        q = torch.zeros(xb.shape, dtype=torch.uint8, device="cuda")
        fog.quantize(xd, fp8.E4M3, s, q=q)
        a = scaling.amax(xb)
        rho, rinv = scaling.compute_scale(a, fp8.E4M3)
        assert np.float32(am.item()) == a and np.float32(s.item()) == rho and np.float32(si.item()) == rinv
        assert np.array_equal(q.cpu().numpy(), scaling.quantize(xb, rho, fp8.E4M3))


def test_argument_errors():
    lib = fog.load()
    st = torch.cuda.current_stream().cuda_stream
    x = torch.zeros(64, dtype=torch.int16, device="cuda")
    out = torch.zeros(1, device="cuda")
    assert lib.fog_amax(x.data_ptr(), 64, None, st) == 1
    assert lib.fog_amax(x.data_ptr(), -1, out.data_ptr(), st) == 2
    assert lib.fog_amax(x.data_ptr() + 2, 8, out.data_ptr(), st) == 3
    q = torch.zeros(64, dtype=torch.uint8, device="cuda")
    assert lib.fog_quantize(x.data_ptr(), 4, 16, 8, 0, out.data_ptr(), q.data_ptr(), 16, None, 0, None, st) == 2
    assert lib.fog_quantize(x.data_ptr(), 4, 16, 16, 0, out.data_ptr(), None, 0, None, 0, None, st) == 1
    assert lib.fog_quantize(x.data_ptr(), 4, 16, 16, 7, out.data_ptr(), q.data_ptr(), 16, None, 0, None, st) == 4
    assert lib.fog_scale(None, 0, 0, out.data_ptr(), None, st) == 1


@pytest.mark.parametrize("fmt", [fp8.E4M3, fp8.E5M2])
@pytest.mark.parametrize("rows,cols,pad,transpose", [
    (256, 512, 0, True), (128, 1024, 0, False), (272, 336, 0, True), (33, 100, 0, True), (5, 17, 3, False),
    (64, 128, 16, True), (1, 8, 0, False), (2048, 4096, 0, True), (0, 64, 0, False)])
def test_quantize_jit_matches_oracle_and_separate_calls(fmt, rows, cols, pad, transpose):
    """The one-call just-in-time flow: abs-max, scale, 1/scale and codes equal the oracle's bit for bit;
    the workspace needs no initialisation and is reused (three calls, one workspace, garbage at the start)."""
    rng = np.random.default_rng(rows * 7 + cols + fmt)
    ws = torch.full((fog.quantize_jit_workspace() // 4,), 0x7F7FFFFF, dtype=torch.int32, device="cuda")
    for call in range(3):
        x = (rng.standard_normal((rows, cols + pad)) * 10.0 ** rng.uniform(-3, 3)).astype(np.float32)
        if rows and call == 1:
            x[rows // 2, cols // 3] = -7.5e4                   # the maximum sits in the last-but-one call only
        xb = synth.f32_to_bf16_bits(x)
        xd = dev(xb)[:, :cols] if pad else dev(xb)
        am, s, si = (torch.full((1,), -1.0, device="cuda") for _ in range(3))
        q = torch.full((rows, cols), 0xAA, dtype=torch.uint8, device="cuda")
        qT = torch.full((cols, rows), 0xAA, dtype=torch.uint8, device="cuda") if transpose else None
        fog.quantize_jit(xd, fmt, am, s, si, ws, q=q, qT=qT)
        torch.cuda.synchronize()
        view = xb[:, :cols]
        a = scaling.amax(view) if rows else np.float32(0.0)
        rho, rinv = scaling.compute_scale(a, fmt)
        assert np.float32(am.item()).tobytes() == np.float32(a).tobytes()
        assert np.float32(s.item()).tobytes() == rho.tobytes() and np.float32(si.item()).tobytes() == rinv.tobytes()
        if rows:
            want = scaling.quantize(view, rho, fmt)
            assert np.array_equal(q.cpu().numpy(), want)
            if transpose:
                assert np.array_equal(qT.cpu().numpy(), want.T)


def test_quantize_jit_argument_errors():
    lib = fog.load()
    st = torch.cuda.current_stream().cuda_stream
    x = torch.zeros((16, 16), dtype=torch.int16, device="cuda")
    q = torch.zeros((16, 16), dtype=torch.uint8, device="cuda")
    f = torch.zeros(3, device="cuda")
    ws = torch.zeros(1024, dtype=torch.int32, device="cuda")
    a, s, si = f.data_ptr(), f.data_ptr() + 4, f.data_ptr() + 8
    call = lambda *args: lib.fog_quantize_jit(*args)
    assert lib.fog_quantize_jit_workspace() == 4096
    assert call(x.data_ptr(), 16, 16, 16, 0, 0, q.data_ptr(), 16, None, 0, a, s, si, ws.data_ptr(), 4000, st) == 5
    assert call(x.data_ptr(), 16, 16, 16, 0, 0, q.data_ptr(), 16, None, 0, a, s, si, None, 4096, st) == 1
    assert call(x.data_ptr(), 16, 16, 16, 0, 0, None, 0, None, 0, a, s, si, ws.data_ptr(), 4096, st) == 1
    assert call(x.data_ptr(), 16, 16, 8, 0, 0, q.data_ptr(), 16, None, 0, a, s, si, ws.data_ptr(), 4096, st) == 2
    assert call(x.data_ptr(), 16, 16, 16, 7, 0, q.data_ptr(), 16, None, 0, a, s, si, ws.data_ptr(), 4096, st) == 4
    assert call(x.data_ptr(), 16, 16, 16, 0, 99, q.data_ptr(), 16, None, 0, a, s, si, ws.data_ptr(), 4096, st) == 2
    assert call(x.data_ptr(), 16, 16, 16, 0, 0, q.data_ptr(), 16, None, 0, a, s, None, ws.data_ptr(), 4096, st) == 0
    torch.cuda.synchronize()


def test_delayed_scaling_flows_of_the_block_driver():
    """Cast.run_delayed (one launch per cast) and Cast.run_delayed_two_calls over five passes with changing data:
    the scale of pass t comes from the history of the abs-maxes of passes < t (1 before any exists), the codes are
    the cast with that scale, the abs-max of pass t reaches the history at pass t + 1; all bit for bit against the
    oracle's history functions (Appendix E)."""
    from paper_2505_20524_amd import block
    rng = np.random.default_rng(77)
    rows, cols = 96, 160
    for one_launch in (True, False):
        for fmt, transpose in ((fp8.E4M3, True), (fp8.E5M2, False)):
            xb0 = synth.f32_to_bf16_bits(rng.standard_normal((rows, cols)).astype(np.float32))
            c = block.Cast(dev(xb0), fmt, transpose)
            hist = np.zeros(1024, np.float32)
            prev_amax = np.float32(0.0)
            for t, gain in enumerate((1.0, 30.0, 0.01, 5.0, 5.0)):
                xb = synth.f32_to_bf16_bits(rng.standard_normal((rows, cols)).astype(np.float32) * gain)
                c.x.copy_(dev(xb))
                c.run_delayed() if one_launch else c.run_delayed_two_calls()
                torch.cuda.synchronize()
                if one_launch:
                    hist[t % 1024] = prev_amax                      # a ring: the oldest entry is replaced
                    assert np.float32(c.amax.item()) == prev_amax     # amax_prev output
                else:
                    hist = scaling.history_update(hist, prev_amax)    # newest first, everything shifts
                rho, rinv = scaling.history_scale(hist, fmt)
                assert np.float32(c.scale.item()).tobytes() == rho.tobytes(), t
                assert np.float32(c.sinv.item()).tobytes() == rinv.tobytes(), t
                want = scaling.quantize(xb, rho, fmt)
                assert np.array_equal(c.q.cpu().numpy(), want), t
                if transpose:
                    assert np.array_equal(c.qT.cpu().numpy(), want.T), t
                prev_amax = scaling.amax(xb)
                if one_launch:
                    am = torch.full((1,), -1.0, device="cuda")
                    fog.delayed_amax(c.state, t, am)
                    assert np.float32(am.item()) == prev_amax
                else:
                    assert np.float32(c.amax.item()) == prev_amax
                assert np.array_equal(c.history.cpu().numpy(), hist)
            # after the small third pass the scale still comes from the large second one: the history remembers
            assert hist.max() == hist[2]


@pytest.mark.parametrize("rows,cols,pad,transpose", [(64, 256, 0, False), (256, 384, 0, True), (37, 100, 4, True), (1500, 4096, 0, False),
                                                     (2048, 2048, 0, True), (2048, 8192, 0, False), (4096, 4608, 0, True)])
def test_quantize_delayed_short_history_forgets(rows, cols, pad, transpose):
    """fog_quantize_delayed with a history of three entries over eight calls (one of them on an empty tensor): an old
    large abs-max leaves the ring after three further calls; row-major, transposing and element-wise kernels, grids
    above and below the 1024 slots of the state."""
    rng = np.random.default_rng(rows + cols)
    fmt = fp8.E4M3 if rows % 2 == 0 else fp8.E5M2
    hist_d = torch.zeros(3, device="cuda")
    state = torch.zeros(fog.quantize_delayed_state(), dtype=torch.uint8, device="cuda")
    s, si, ap = (torch.zeros(1, device="cuda") for _ in range(3))
    ring = np.zeros(3, np.float32)
    prev = np.float32(0.0)
    for t, gain in enumerate((1.0, 100.0, 1.0, 0.5, None, 2.0, 1.0, 1.0)):
        ring[t % 3] = prev
        rho, rinv = scaling.history_scale(ring, fmt, margin=1)
        if gain is None:     # an empty tensor: the history advances, nothing is cast
            fog.quantize_delayed(torch.zeros((0, cols), dtype=torch.int16, device="cuda"), fmt, hist_d, t, state, s, si, amax_prev=ap,
                                 margin=1)
            torch.cuda.synchronize()
            prev_next = np.float32(0.0)
        else:
            xb = synth.f32_to_bf16_bits(rng.standard_normal((rows, cols + pad)).astype(np.float32) * gain)
            x = dev(xb)[:, :cols] if pad else dev(xb)
            q = torch.full((rows, cols), 0xAA, dtype=torch.uint8, device="cuda")
            qT = torch.full((cols, rows), 0xAA, dtype=torch.uint8, device="cuda") if transpose else None
            fog.quantize_delayed(x, fmt, hist_d, t, state, s, si, q=q, qT=qT, amax_prev=ap, margin=1)
            torch.cuda.synchronize()
            want = scaling.quantize(xb[:, :cols], rho, fmt)
            assert np.array_equal(q.cpu().numpy(), want), t
            if transpose:
                assert np.array_equal(qT.cpu().numpy(), want.T), t
            prev_next = scaling.amax(xb[:, :cols])
        assert np.float32(s.item()).tobytes() == rho.tobytes(), t
        assert np.float32(si.item()).tobytes() == rinv.tobytes(), t
        assert np.float32(ap.item()) == prev
        assert np.array_equal(hist_d.cpu().numpy(), ring)
        prev = prev_next
    # the abs-max of the gain-100 pass (t = 1) entered at t = 2 and was replaced at t = 5
    assert ring.max() < 20.0


def test_quantize_delayed_argument_errors():
    lib = fog.load()
    st = torch.cuda.current_stream().cuda_stream
    x = torch.zeros((4, 64), dtype=torch.int16, device="cuda")
    q = torch.zeros((4, 64), dtype=torch.uint8, device="cuda")
    h = torch.zeros(8, device="cuda")
    state = torch.zeros(fog.quantize_delayed_state(), dtype=torch.uint8, device="cuda")
    f = fscalar(1.0)
    ok = [x.data_ptr(), 4, 64, 64, 0, 0, h.data_ptr(), 8, 0, state.data_ptr(), state.numel(), q.data_ptr(), 64, None, 0, None, f.data_ptr(),
          None, st]

    def with_(i, v):
        t = list(ok)
        t[i] = v
        return lib.fog_quantize_delayed(*t)
    assert lib.fog_quantize_delayed(*ok) == 0
    assert with_(6, None) == 1 and with_(9, None) == 1 and with_(16, None) == 1 and with_(0, None) == 1 and with_(11, None) == 1
    assert with_(7, 0) == 2 and with_(8, -1) == 2 and with_(5, 100) == 2 and with_(3, 32) == 2
    assert with_(9, state.data_ptr() + 1) == 3 and with_(0, x.data_ptr() + 1) == 3
    assert with_(4, 2) == 4
    assert with_(10, 100) == 5
    assert lib.fog_delayed_amax(None, 0, f.data_ptr(), st) == 1 and lib.fog_delayed_amax(state.data_ptr(), -1, f.data_ptr(), st) == 2
    torch.cuda.synchronize()


def test_block_driver_jit_cast_equals_the_three_separate_calls():
    """Cast.run (fog_quantize_jit, two launches) and Cast.run_separate (fog_amax, fog_scale, fog_quantize) give the
    same bytes and scalars, bit for bit."""
    from paper_2505_20524_amd import block
    rng = np.random.default_rng(3)
    xb = synth.f32_to_bf16_bits(rng.standard_normal((256, 384)).astype(np.float32) * 7)
    for fmt, transpose in ((fp8.E4M3, True), (fp8.E5M2, False)):
        a, b = block.Cast(dev(xb), fmt, transpose), block.Cast(dev(xb), fmt, transpose)
        a.run()
        b.run_separate()
        torch.cuda.synchronize()
        assert torch.equal(a.q, b.q) and (not transpose or torch.equal(a.qT, b.qT))
        for u, v in ((a.amax, b.amax), (a.scale, b.scale), (a.sinv, b.sinv)):
            assert np.float32(u.item()).tobytes() == np.float32(v.item()).tobytes()
        rho, _ = scaling.compute_scale(scaling.amax(xb), fmt)
        assert np.array_equal(a.q.cpu().numpy(), scaling.quantize(xb, rho, fmt))


@pytest.mark.parametrize("shapes", [[(1, 16)], [(64, 256), (8, 48)], [(300, 1024), (2, 8), (128, 4096)],
                                    [(2048, 4096), (96, 160), (5000, 1024), (1, 16)], [(4100, 8192), (333, 1008)],
                                    [(64 + 16 * k, 128 + 32 * (k % 5)) for k in range(19)] + [(3000, 2048)],     # a whole step's tensors in one call
                                    [(16, 16 + 16 * k) for k in range(32)]])                                        # the most jobs a call takes
def test_quantize_jit_batch_equals_the_single_tensor_call(shapes):
    """fog_quantize_jit_batch (two launches for up to 32 tensors) against fog_quantize_jit per tensor and against the
    oracle: bytes, abs-max, scale and reciprocal scale bit for bit; mixed formats, sizes from 16 elements to more than
    the largest grids take in one trip."""
    rng = np.random.default_rng(len(shapes) * 100 + shapes[0][0])
    items, refs = [], []
    for k, (rows, cols) in enumerate(shapes):
        fmt = fp8.E4M3 if k % 2 == 0 else fp8.E5M2
        xb = synth.f32_to_bf16_bits(rng.standard_normal((rows, cols)).astype(np.float32) * (10.0 ** (k % 7 - 1)))
        x = dev(xb)
        q = torch.full((rows, cols), 0xAA, dtype=torch.uint8, device="cuda")
        am, sc, si = (torch.full((1,), -1.0, device="cuda") for _ in range(3))
        items.append((x, fmt, q, am, sc, si))
        refs.append((xb, fmt))
    ws = torch.full((fog.quantize_jit_batch_workspace(len(items)) // 4,), 0x7F7FFFFF, dtype=torch.int32, device="cuda")   # garbage on entry
    fog.quantize_jit_batch(fog.make_cast_jobs(items, margin=1), ws)
    torch.cuda.synchronize()
    one_ws = torch.empty(fog.quantize_jit_workspace(), dtype=torch.uint8, device="cuda")
    for (x, fmt, q, am, sc, si), (xb, _) in zip(items, refs):
        a = scaling.amax(xb)
        rho, rinv = scaling.compute_scale(a, fmt, margin=1)
        assert np.float32(am.item()) == a
        assert np.float32(sc.item()).tobytes() == rho.tobytes() and np.float32(si.item()).tobytes() == rinv.tobytes()
        assert np.array_equal(q.cpu().numpy(), scaling.quantize(xb, rho, fmt))
        q1 = torch.empty_like(q)
        am1, sc1, si1 = (torch.zeros(1, device="cuda") for _ in range(3))
        fog.quantize_jit(x, fmt, am1, sc1, si1, one_ws, q=q1, margin=1)
        torch.cuda.synchronize()
        assert torch.equal(q, q1) and am1.item() == am.item() and sc1.item() == sc.item() and si1.item() == si.item()


def test_quantize_jit_batch_argument_errors():
    lib = fog.load()
    st = torch.cuda.current_stream().cuda_stream
    x = torch.zeros((4, 64), dtype=torch.int16, device="cuda")
    q = torch.zeros((4, 64), dtype=torch.uint8, device="cuda")
    f = [torch.zeros(1, device="cuda") for _ in range(3)]
    ws = torch.zeros(33 * 4096, dtype=torch.uint8, device="cuda")

    def call(items, count=None, wsp=ws.data_ptr(), wsb=ws.numel(), **over):
        jobs = fog.make_cast_jobs(items)
        for k, v in over.items():
            setattr(jobs[0], k, v)
        import ctypes
        return lib.fog_quantize_jit_batch(ctypes.cast(jobs, ctypes.c_void_p), len(items) if count is None else count, wsp, wsb, st)
    good = (x, fp8.E4M3, q, f[0], f[1], f[2])
    assert call([good]) == 0 and call([good], scale_inv=None) == 0 and call([], count=0) == 0
    assert call([good], wsp=None) == 1 and call([good], x_bf16=None) == 1 and call([good], q=None) == 1 and call([good], amax=None) == 1
    assert call([good] * 33) == 2 and call([good], rows=0) == 2 and call([good], margin=100) == 2
    assert call([good], x_bf16=x.data_ptr() + 2) == 3 and call([good], wsp=ws.data_ptr() + 1) == 3
    assert call([good], fmt=2) == 4 and call([good], cols=63) == 4
    assert call([good, good], wsb=4096) == 5
    torch.cuda.synchronize()


def _with_non_finite(rows, cols, seed):
    """bf16 bits of a normal matrix with NaN (both signs, a payload) and infinities planted at edge and interior places."""
    rng = np.random.default_rng(seed)
    xb = synth.f32_to_bf16_bits(rng.standard_normal((rows, cols)).astype(np.float32) * 5)
    flat = xb.reshape(-1)
    n = flat.size
    spots = {0: 0x7FC0, n - 1: 0xFFC0, n // 2: 0x7F80, n // 3: 0xFF80, min(n - 1, 17): 0x7FA5, min(n - 1, 16 * 9 + 3): 0xFFFF}
    for pos, bits in spots.items():
        flat[pos] = bits
    return xb


@pytest.mark.parametrize("fmt", [fp8.E4M3, fp8.E5M2])
@pytest.mark.parametrize("rows,cols,tr", [(64, 256, False), (256, 384, True), (33, 17, True), (1, 16, False), (1500, 1024, False)])
def test_non_finite_inputs_keep_their_meaning(fmt, rows, cols, tr):
    """NaN inputs become the format's NaN code with the input's sign and infinities saturate, exactly as the
    oracle's cast defines them, on every cast path (rows, fused transpose, general, and the batched call);
    the abs-max of such a tensor is not finite, so its scale is 1 by the scale rule."""
    xb = _with_non_finite(rows, cols, rows + cols)
    xd = dev(xb)
    for rho in (1.0, 37.5):
        want = scaling.quantize(xb, np.float32(rho), fmt)
        assert (want == 0x7F).any() and (want == 0xFF).any()          # the oracle did produce NaN codes of both signs
        q = torch.full((rows, cols), 0x55, dtype=torch.uint8, device="cuda")
        qT = torch.full((cols, rows), 0x55, dtype=torch.uint8, device="cuda") if tr else None
        am = torch.full((1,), -1.0, device="cuda")
        fog.quantize(xd, fmt, fscalar(rho), q=q, qT=qT, amax_out=am)
        assert np.array_equal(q.cpu().numpy(), want), rho
        if tr:
            assert np.array_equal(qT.cpu().numpy(), want.T)
        assert np.isnan(am.item()) and np.isnan(scaling.amax(xb))
    assert np.isnan(gpu_amax(xb))
    # the one-call just-in-time cast: abs-max NaN -> scale 1 (the rule for a non-finite abs-max)
    am, sc, si = (torch.full((1,), -1.0, device="cuda") for _ in range(3))
    ws = torch.empty(fog.quantize_jit_workspace(), dtype=torch.uint8, device="cuda")
    q = torch.full((rows, cols), 0x55, dtype=torch.uint8, device="cuda")
    fog.quantize_jit(xd, fmt, am, sc, si, ws, q=q)
    rho, rinv = scaling.compute_scale(scaling.amax(xb), fmt)
    assert rho == 1.0 and np.float32(sc.item()) == rho and np.float32(si.item()) == rinv
    assert np.array_equal(q.cpu().numpy(), scaling.quantize(xb, rho, fmt))
    if (rows * cols) % 16 == 0:
        q2 = torch.full((rows, cols), 0x55, dtype=torch.uint8, device="cuda")
        jobs = fog.make_cast_jobs([(xd, fmt, q2, am, sc, si)])
        wsb = torch.empty(fog.quantize_jit_batch_workspace(1), dtype=torch.uint8, device="cuda")
        fog.quantize_jit_batch(jobs, wsb)
        assert np.array_equal(q2.cpu().numpy(), scaling.quantize(xb, rho, fmt))
        assert np.float32(sc.item()) == 1.0


def test_only_infinities_saturate_and_give_scale_one():
    xb = synth.f32_to_bf16_bits(np.linspace(-3, 3, 64 * 32, dtype=np.float32).reshape(64, 32))
    xb[5, 7] = 0x7F80
    xb[60, 0] = 0xFF80
    for fmt in (fp8.E4M3, fp8.E5M2):
        q = torch.zeros((64, 32), dtype=torch.uint8, device="cuda")
        fog.quantize(dev(xb), fmt, fscalar(2.0), q=q)
        got = q.cpu().numpy()
        assert np.array_equal(got, scaling.quantize(xb, np.float32(2.0), fmt))
        top = 0x7E if fmt == fp8.E4M3 else 0x7B
        assert got[5, 7] == top and got[60, 0] == (top | 0x80)
    assert gpu_amax(xb) == np.float32(np.inf)


def test_quantize_delayed_batch_equals_the_calls_one_by_one_and_the_oracle():
    """fog_quantize_delayed_batch over six steps with changing data: three tensors of different sizes, formats and history
    lengths in one launch; scales, codes, previous abs-maxes and histories bit for bit against the oracle's history
    functions (Appendix E) and against fog_quantize_delayed on a second set of states."""
    rng = np.random.default_rng(2024)
    specs = [(64, 256, fp8.E4M3, 1024), (1500, 4096, fp8.E5M2, 3), (333, 48, fp8.E4M3, 2)]   # the second spans more workgroups than state slots
    dst = fog.quantize_delayed_state()
    T = []
    for rows, cols, fmt, hl in specs:
        T.append(dict(rows=rows, cols=cols, fmt=fmt, x=torch.zeros((rows, cols), dtype=torch.int16, device="cuda"),
                      q=torch.full((rows, cols), 0xAA, dtype=torch.uint8, device="cuda"),
                      q1=torch.full((rows, cols), 0xAA, dtype=torch.uint8, device="cuda"),
                      hist=torch.zeros(hl, device="cuda"), hist1=torch.zeros(hl, device="cuda"),
                      state=torch.zeros(dst, dtype=torch.uint8, device="cuda"), state1=torch.zeros(dst, dtype=torch.uint8, device="cuda"),
                      ap=torch.full((1,), -1.0, device="cuda"), s=torch.zeros(1, device="cuda"), si=torch.zeros(1, device="cuda"),
                      ap1=torch.full((1,), -1.0, device="cuda"), s1=torch.zeros(1, device="cuda"), si1=torch.zeros(1, device="cuda"),
                      ring=np.zeros(hl, np.float32), prev=np.float32(0.0)))
    jobs = fog.make_delayed_jobs([(t["x"], t["fmt"], t["q"], t["hist"], t["state"], t["ap"], t["s"], t["si"]) for t in T], margin=1)
    for step, gain in enumerate((1.0, 80.0, 0.02, 3.0, 3.0, 0.5)):
        xbs = []
        for k, t in enumerate(T):
            xb = synth.f32_to_bf16_bits(rng.standard_normal((t["rows"], t["cols"])).astype(np.float32) * gain * (k + 1))
            t["x"].copy_(dev(xb))
            xbs.append(xb)
        fog.quantize_delayed_batch(jobs, step)
        for t in T:
            fog.quantize_delayed(t["x"], t["fmt"], t["hist1"], step, t["state1"], t["s1"], t["si1"], q=t["q1"], amax_prev=t["ap1"], margin=1)
        torch.cuda.synchronize()
        for t, xb in zip(T, xbs):
            hl = t["ring"].size
            t["ring"][step % hl] = t["prev"]
            rho, rinv = scaling.history_scale(t["ring"], t["fmt"], margin=1)
            assert np.float32(t["s"].item()).tobytes() == rho.tobytes(), step
            assert np.float32(t["si"].item()).tobytes() == rinv.tobytes(), step
            assert np.float32(t["ap"].item()) == t["prev"]
            assert np.array_equal(t["hist"].cpu().numpy(), t["ring"])
            assert np.array_equal(t["q"].cpu().numpy(), scaling.quantize(xb, rho, t["fmt"])), step
            for a, b in (("q", "q1"), ("s", "s1"), ("si", "si1"), ("ap", "ap1"), ("hist", "hist1"), ("state", "state1")):
                assert torch.equal(t[a], t[b]), (step, a)
            t["prev"] = scaling.amax(xb)
            am = torch.full((1,), -1.0, device="cuda")
            fog.delayed_amax(t["state"], step, am)
            assert np.float32(am.item()) == t["prev"]
    # argument errors: nothing is launched
    lib = fog.load()
    st = torch.cuda.current_stream().cuda_stream
    import ctypes as C
    call = lib.fog_quantize_delayed_batch
    ptr = C.cast(jobs, C.c_void_p)
    assert call(ptr, 0, 0, st) == 0
    assert call(None, 3, 0, st) == 1
    assert call(ptr, 33, 0, st) == 2
    assert call(ptr, 3, -1, st) == 2
    before = [t["q"].clone() for t in T]
    bad = fog.make_delayed_jobs([(T[0]["x"], T[0]["fmt"], T[0]["q"], T[0]["hist"], T[0]["state"][:64], None, T[0]["s"], None)])
    assert call(C.cast(bad, C.c_void_p), 1, 6, st) == 5
    bad = fog.make_delayed_jobs([(T[0]["x"][:, :8], T[0]["fmt"], T[0]["q"][:, :8], T[0]["hist"], T[0]["state"], None, T[0]["s"], None)])
    bad[0].rows, bad[0].cols = 1, 8
    assert call(C.cast(bad, C.c_void_p), 1, 6, st) == 4
    bad = fog.make_delayed_jobs([(T[0]["x"], 7, T[0]["q"], T[0]["hist"], T[0]["state"], None, T[0]["s"], None)])
    assert call(C.cast(bad, C.c_void_p), 1, 6, st) == 4
    bad = fog.make_delayed_jobs([(T[0]["x"], T[0]["fmt"], T[0]["q"], T[0]["hist"], T[0]["state"], None, T[0]["s"], None)])
    bad[0].scale = None
    assert call(C.cast(bad, C.c_void_p), 1, 6, st) == 1
    torch.cuda.synchronize()
    assert all(torch.equal(a, t["q"]) for a, t in zip(before, T))

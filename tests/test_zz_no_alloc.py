"""GPU: the attention backward that takes no workspace (fog_fp8_attn_bwd_static) against fog_fp8_attn_bwd.

The two entry points run the same kernels; the only difference is where the per-row constants live (the
library's own device array instead of a caller workspace), so every output must agree bit for bit.
Two calls in a row on the same GPU share the array: the second, smaller, call must not see anything of
the first.  Each call goes through the C ABI (ctypes), with every buffer allocated beforehand.
"""
import math

import numpy as np
import pytest
import torch

from oracle import attention, bf16, fp8, scaling
from paper_2505_20524_amd import fog, synth
from parity import dev, fscalar, host_u16

pytestmark = pytest.mark.gpu


def _case(seed, B, H, Hkv, S):
    """Device-resident inputs of one backward call: casts and the forward's O / lse from the oracle-free GPU forward."""
    q, _, _, do = synth.small_attention(seed, B, H, S)
    _, k, v, _ = synth.small_attention(seed + 1, B, Hkv, S)
    c = {}
    for name, t, fmt in (("q", q, fp8.E4M3), ("k", k, fp8.E4M3), ("v", v, fp8.E4M3), ("do", do, fp8.E5M2)):
        rho, rinv = scaling.compute_scale(scaling.amax(t), fmt)
        c[name] = (dev(scaling.quantize(t.reshape(-1, 128), rho, fmt).reshape(t.shape)), fscalar(rinv))
    s = 1.0 / math.sqrt(128)
    O = torch.empty((B, H, S, 128), dtype=torch.int16, device="cuda")
    lse = torch.empty((B, H, S), device="cuda")
    fog.fp8_attn_fwd(B, H, S, 128, s, True, c["q"][0], c["k"][0], c["v"][0], c["q"][1], c["k"][1], c["v"][1], fscalar(448.0),
                     O, lse, H_kv=Hkv)
    return dict(B=B, H=H, Hkv=Hkv, S=S, s=s, c=c, O=O, lse=lse, dO=dev(do), rho_p=fscalar(448.0), rho_ds=fscalar(2.0 ** 18))


def _outputs(k):
    B, H, Hkv, S = k["B"], k["H"], k["Hkv"], k["S"]
    dQ = torch.full((B, H, S, 128), 0x7FC0, dtype=torch.int16, device="cuda")
    dK, dV = (torch.full((B, Hkv, S, 128), 0x7FC0, dtype=torch.int16, device="cuda") for _ in range(2))
    return dQ, dK, dV, torch.full((1,), -1.0, device="cuda")


def _args(k, outs):
    c = k["c"]
    return (k["B"], k["H"], k["S"], 128, k["s"], True, c["q"][0], c["k"][0], c["v"][0], c["q"][1], c["k"][1], c["v"][1],
            k["O"], k["dO"], c["do"][0], c["do"][1], k["lse"], k["rho_p"], k["rho_ds"], outs[0], outs[1], outs[2])


def test_static_scratch_backward_equals_the_workspace_backward_on_two_calls_in_a_row():
    # first call: grouped queries, 2 x 4 heads of 320 tokens; second call: smaller (1 x 2 heads of 128 tokens)
    cases = [_case(7100, 2, 4, 2, 320), _case(7200, 1, 2, 2, 128)]
    want = []
    for k in cases:                                   # the existing entry point, with a caller workspace
        outs = _outputs(k)
        ws = torch.empty(fog.fp8_attn_workspace(k["B"], k["H"], k["S"], 128, True, H_kv=k["Hkv"]), dtype=torch.uint8, device="cuda")
        fog.fp8_attn_bwd(*_args(k, outs), amax_ds=outs[3], workspace=ws, H_kv=k["Hkv"])
        torch.cuda.synchronize()
        want.append([host_u16(t) for t in outs[:3]] + [outs[3].item()])
        assert want[-1][3] > 0 and all(np.isfinite(bf16.bits_to_f64(w)).all() for w in want[-1][:3])
    got_outs = [_outputs(k) for k in cases]          # every buffer exists before the calls under test
    torch.cuda.synchronize()
    for k, outs in zip(cases, got_outs):              # back to back on one stream, no allocation in between
        fog.fp8_attn_bwd_static(*_args(k, outs), amax_ds=outs[3], H_kv=k["Hkv"])
    torch.cuda.synchronize()
    for k, outs, w in zip(cases, got_outs, want):
        for name, t, ref in zip(("dQ", "dK", "dV"), outs[:3], w[:3]):
            assert np.array_equal(host_u16(t), ref), "%s differs (B=%d H=%d S=%d)" % (name, k["B"], k["H"], k["S"])
        assert outs[3].item() == w[3]


def test_static_scratch_backward_against_the_oracle_and_its_size_limit():
    """One head of the second call's shape against the float64 oracle (the same gate as the workspace
    entry point), and the stated limit: one row more than the array holds is refused before any launch."""
    k = _case(7300, 1, 1, 1, 128)
    outs = _outputs(k)
    fog.fp8_attn_bwd_static(*_args(k, outs), amax_ds=outs[3])
    torch.cuda.synchronize()
    c = k["c"]
    h = lambda t: t.cpu().numpy()
    head = (h(c["q"][0])[0, 0], h(c["k"][0])[0, 0], h(c["v"][0])[0, 0], np.float32(c["q"][1].item()), np.float32(c["k"][1].item()),
            np.float32(c["v"][1].item()))
    tail = (host_u16(k["O"])[0, 0], host_u16(k["dO"])[0, 0], h(c["do"][0])[0, 0], np.float32(c["do"][1].item()), h(k["lse"])[0, 0],
            k["s"], 448.0, 2.0 ** 18, True)
    r = attention.attn_bwd_head(*head, *tail)
    from parity import check_attention
    from mfma_model import bwd_cast_slack
    sl = bwd_cast_slack(*head, *tail)
    for name, t, ref, s_ in zip(("dQ", "dK", "dV"), outs[:3], r[:3], sl):
        check_attention(host_u16(t)[0, 0], ref, s_, what=name)
    lib = fog.load()
    S_big = 64 * ((fog.ATTN_BWD_STATIC_MAX_ROWS // 64) + 1)
    before = [host_u16(t).copy() for t in outs[:3]]
    a = _args(k, outs)
    st = lib.fog_fp8_attn_bwd_static(1, 1, 1, S_big, 128, k["s"], 1, *[x.data_ptr() for x in a[6:]], None,
                                     torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert st == 5
    assert all(np.array_equal(host_u16(t), b) for t, b in zip(outs[:3], before))

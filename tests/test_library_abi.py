"""The built C-ABI library loads and exports every symbol the header declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "fog.h")
LIB = os.path.join(ROOT, "paper_2505_20524_amd", "libfog.so")


def declared_symbols(header=HEADER):
    text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(fog_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_hot_path_calls():
    names = declared_symbols()
    for need in ("fog_amax", "fog_scale", "fog_quantize", "fog_fp8_gemm", "fog_fp8_attn_fwd", "fog_fp8_attn_bwd"):
        assert need in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        pytest.fail("libfog.so missing: run `python __graft_entry__.py` before the tests")
    lib = ctypes.CDLL(LIB)
    for name in declared_symbols():
        assert hasattr(lib, name), name
    for name in declared_symbols(os.path.join(ROOT, "include", "fog_probe.h")):     # the benchmark's measurement helpers
        assert hasattr(lib, name), name
    lib.fog_status_string.restype = ctypes.c_char_p
    assert lib.fog_status_string(0) == b"ok"
    assert lib.fog_version() >= 100


def test_binding_covers_the_header_and_pure_host_queries():
    from paper_2505_20524_amd import fog
    assert sorted(fog.SIGNATURES) == declared_symbols()
    lib = fog.load()
    assert lib.fog_fp8_gemm_workspace(0, 4096, 8192, 2048) == 0              # 512 tiles: no split
    assert lib.fog_fp8_gemm_workspace(2, 2048, 2048, 16384) % (256 * 256 * 4) == 0
    assert lib.fog_fp8_attn_workspace(4, 16, 16, 2048, 128, 1) >= 4 * 16 * 2048 * 4
    assert lib.fog_fp8_attn_workspace(4, 16, 16, 2048, 128, 0) == 0

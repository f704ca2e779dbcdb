"""Pins for the oracle's FP8 codec and bf16 helpers (CPU only)."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import bf16, fp8

FMTS = [fp8.E4M3, fp8.E5M2]
TORCH = {fp8.E4M3: torch.float8_e4m3fn, fp8.E5M2: torch.float8_e5m2}
HERE = os.path.dirname(__file__)


def finite_codes(fmt):
    c = np.arange(256, dtype=np.uint8)
    return c[np.isfinite(fp8.decode(c, fmt))]


def brute_encode(values, fmt):
    """Nearest finite code by exhaustive search in exact arithmetic; ties -> even code; saturating."""
    codes = finite_codes(fmt)
    pos = codes[codes < 0x80]
    grid = [(Fraction(float(fp8.decode(np.uint8(c), fmt))), int(c)) for c in pos]
    out = []
    for v in values:
        v = float(v)
        if math.isnan(v):
            out.append(0x7F | (0x80 if math.copysign(1, v) < 0 else 0))
            continue
        sign = 0x80 if math.copysign(1.0, v) < 0 else 0
        if math.isinf(v):
            out.append(grid[-1][1] | sign)
            continue
        a = Fraction(abs(v))
        best, bestd = None, None
        for g, c in grid:
            d = abs(g - a)
            if bestd is None or d < bestd or (d == bestd and (c & 1) == 0 and (best & 1) == 1):
                best, bestd = c, d
        out.append(best | sign)
    return np.array(out, dtype=np.uint8)


def test_golden_points():
    name = {"E4M3": fp8.E4M3, "E5M2": fp8.E5M2}
    n = 0
    for line in open(os.path.join(HERE, "golden", "fp8_format_points.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f, code, val = line.split()
        got = float(fp8.decode(np.uint8(int(code, 16)), name[f]))
        want = float(val)
        if math.isnan(want):
            assert math.isnan(got)
        else:
            assert got == want and math.copysign(1, got) == math.copysign(1, want), line
        n += 1
    assert n >= 25
    assert fp8.fp8_max(fp8.E4M3) == 448.0 and fp8.fp8_max(fp8.E5M2) == 57344.0


@pytest.mark.parametrize("fmt", FMTS)
def test_decode_matches_library_and_is_monotone(fmt):
    c = np.arange(256, dtype=np.uint8)
    mine = fp8.decode(c, fmt)
    lib = torch.from_numpy(c.copy()).view(TORCH[fmt]).to(torch.float64).numpy()
    assert np.array_equal(np.isnan(mine), np.isnan(lib))
    ok = ~np.isnan(mine)
    assert np.array_equal(mine[ok], lib[ok])
    pos = mine[:0x80]
    pos = pos[np.isfinite(pos)]
    assert np.all(np.diff(pos) > 0)
    assert np.array_equal(fp8.decode(c[:0x80] | 0x80, fmt)[np.isfinite(mine[:0x80])], -pos)


@pytest.mark.parametrize("fmt", FMTS)
def test_encode_roundtrip_midpoints_neighbours(fmt):
    codes = finite_codes(fmt)
    vals = fp8.decode(codes, fmt).astype(np.float32)
    assert np.array_equal(fp8.encode_sat(vals, fmt), codes)
    pos = codes[codes < 0x80]
    for c in pos[:-1]:
        lo, hi = float(fp8.decode(c, fmt)), float(fp8.decode(np.uint8(c + 1), fmt))
        mid = np.float32((lo + hi) / 2)
        assert float(mid) == (lo + hi) / 2          # representable in binary32
        even = c if c % 2 == 0 else c + 1
        assert fp8.encode_sat(mid, fmt) == even
        assert fp8.encode_sat(-mid, fmt) == (even | 0x80)
        assert fp8.encode_sat(np.nextafter(mid, np.float32(0)), fmt) == c
        assert fp8.encode_sat(np.nextafter(mid, np.float32(np.inf)), fmt) == c + 1


@pytest.mark.parametrize("fmt", FMTS)
def test_encode_special_values(fmt):
    mx = np.float32(fp8.fp8_max(fmt))
    cmax = 0x7E if fmt == fp8.E4M3 else 0x7B
    for v in [mx, np.nextafter(mx, np.float32(np.inf)), mx * np.float32(1.04), mx * 2, np.float32(1e30), np.float32(np.inf)]:
        assert fp8.encode_sat(np.float32(v), fmt) == cmax
        assert fp8.encode_sat(np.float32(-v), fmt) == (cmax | 0x80)
    assert fp8.encode_sat(np.float32(np.nan), fmt) & 0x7F == 0x7F
    assert fp8.encode_sat(np.float32(0.0), fmt) == 0x00
    assert fp8.encode_sat(np.float32(-0.0), fmt) == 0x80
    tiny = np.float32(fp8.decode(np.uint8(1), fmt) / 2)      # half the smallest subnormal: tie -> 0
    assert fp8.encode_sat(tiny, fmt) == 0x00
    assert fp8.encode_sat(-tiny, fmt) == 0x80
    assert fp8.encode_sat(np.nextafter(tiny, np.float32(1)), fmt) == 0x01
    assert fp8.encode_sat(np.float32(1e-45), fmt) == 0x00      # binary32 subnormal
    assert fp8.encode_sat(np.float32(-1e-40), fmt) == 0x80


@pytest.mark.parametrize("fmt", FMTS)
def test_encode_vs_brute_force_search(fmt):
    rng = np.random.default_rng(7)
    x = (rng.standard_normal(3000) * np.exp(rng.standard_normal(3000) * 6)).astype(np.float32)
    edge = np.array([0, 1e-9, 448, 449, 464, 465, 57344, 61439, 61440, 1e9, np.inf, -np.inf], dtype=np.float32)
    x = np.concatenate([x, edge, -edge])
    assert np.array_equal(fp8.encode_sat(x, fmt), brute_encode(x, fmt))


@pytest.mark.parametrize("fmt", FMTS)
def test_encode_all_bf16_inputs_vs_library(fmt):
    """Every bf16 value (the bulk kernels' whole input domain at rho = 1) and a stratified binary32 sweep."""
    allb = np.arange(65536, dtype=np.uint16)
    x = bf16.bits_to_f32(allb)
    fin = np.isfinite(x)
    mx = fp8.fp8_max(fmt)
    lib = torch.from_numpy(x[fin].copy()).clamp(-mx, mx).to(TORCH[fmt]).view(torch.uint8).numpy()
    assert np.array_equal(fp8.encode_sat(x[fin], fmt), lib)
    # binary32 patterns with every exponent and the top 11 mantissa bits, plus both neighbours
    pat = (np.arange(1 << 20, dtype=np.uint32) << np.uint32(12))
    for delta in (0, 1, 0xFFF, 0x800, 0x7FF, 0x801):
        y = (pat | np.uint32(delta)).view(np.float32)
        y = y[np.isfinite(y)]
        lib = torch.from_numpy(y.copy()).clamp(-mx, mx).to(TORCH[fmt]).view(torch.uint8).numpy()
        assert np.array_equal(fp8.encode_sat(y, fmt), lib)


def test_bf16_helpers():
    allb = np.arange(65536, dtype=np.uint16)
    v = bf16.bits_to_f64(allb)
    fin = np.isfinite(v)
    assert np.array_equal(bf16.f64_to_bits_rne(v[fin]), allb[fin])
    # library agreement on binary32-representable inputs (a single rounding on both sides)
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(200000) * np.exp(rng.standard_normal(200000) * 8)).astype(np.float32)
    lib = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bf16.f64_to_bits_rne(x.astype(np.float64)), lib)
    # midpoints between neighbours go to the even pattern; a hair to either side goes to the nearer
    b = np.arange(0x0001, 0x7F7F, 37, dtype=np.uint16)
    lo, hi = bf16.bits_to_f64(b), bf16.bits_to_f64(b + np.uint16(1))
    mid = (lo + hi) / 2
    even = np.where(b % 2 == 0, b, b + 1).astype(np.uint16)
    assert np.array_equal(bf16.f64_to_bits_rne(mid), even)
    assert np.array_equal(bf16.f64_to_bits_rne(np.nextafter(mid, 0)), b)
    assert np.array_equal(bf16.f64_to_bits_rne(np.nextafter(mid, np.inf)), b + np.uint16(1))
    assert np.array_equal(bf16.f64_to_bits_rne(-mid), even | np.uint16(0x8000))
    assert bf16.f64_to_bits_rne(np.float64(1e39)) == 0x7F80
    assert bf16.half_ulp(np.float64(1.0)) == 2.0 ** -8 and bf16.half_ulp(np.float64(3.0)) == 2.0 ** -7 and bf16.half_ulp(np.float64(1.99)) == 2.0 ** -8

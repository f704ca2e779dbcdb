"""Seeded synthetic inputs with the structure of the paper's activations.

The paper's tensors (activations of trained Llama / FOG models) are not
available; these stand in for them and take their structure from the paper:
per-channel outliers of magnitude tau * sigma (Appendix C, tau-outliers),
"massive activations" on a few channels (Section 2), heavy tails (kurtosis,
Section 4).  Everything is drawn on the host from numpy's PCG64 with a fixed
seed and rounded once to bfloat16; the SAME bf16 bit patterns are handed to the
GPU library and to the CPU oracle, so the generator is not part of parity.

This module holds no arithmetic of the method (no scaling, no FP8, no GEMM).
"""
from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20524 * 10


def f32_to_bf16_bits(x):
    """binary32 -> bfloat16 bit patterns, round-to-nearest-even (finite inputs)."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal(rng, shape, std=1.0):
    return rng.standard_normal(shape, dtype=np.float32) * np.float32(std)


def student_t(rng, shape, nu=3.0, scale=1.0):
    """Heavy-tailed values: normal / sqrt(chi2_nu / nu)."""
    z = rng.standard_normal(shape, dtype=np.float32)
    c = rng.chisquare(nu, size=shape).astype(np.float32)
    return z / np.sqrt(c / np.float32(nu)) * np.float32(scale)


def scale_columns(x, rng, n_cols, factor):
    """Multiply n_cols distinct seeded columns (last axis) by `factor`: channel outliers."""
    cols = rng.choice(x.shape[-1], size=n_cols, replace=False)
    x[..., cols] *= np.float32(factor)
    return cols


@dataclass
class Linear:
    """One linear layer Y = X W^T: X [M,K] activations, W [N,K] weights, dY [M,N] output gradient."""
    name: str
    M: int
    N: int
    K: int


@dataclass
class Attn:
    B: int
    H: int
    S: int
    D: int = 128


@dataclass
class Config:
    cid: int
    label: str
    linears: list = field(default_factory=list)
    attn: Attn = None
    act: str = "normal"          # "normal" | "student_t"
    outlier_cols: int = 0
    outlier_factor: float = 1.0
    grad_std: float = 1e-3
    attn_dist: str = "normal"
    do_std: float = 1e-2
    backward: bool = True


CONFIGS = {
    1: Config(1, "linear fwd 512x1024x1024", [Linear("lin", 512, 1024, 1024)], None,
              outlier_cols=4, outlier_factor=50.0, backward=False),
    2: Config(2, "linear fwd+dgrad+wgrad 4096x8192x2048", [Linear("lin", 4096, 8192, 2048)], None,
              outlier_cols=20, outlier_factor=100.0),
    3: Config(3, "attention fwd+bwd B4 H16 S2048 D128", [], Attn(4, 16, 2048)),
    4: Config(4, "1.5B-scale block: hidden 2048, 16 heads, MLP 8192, 8x2048 tokens",
              [Linear("qkv", 16384, 6144, 2048), Linear("out", 16384, 2048, 2048),
               Linear("up", 16384, 8192, 2048), Linear("down", 16384, 2048, 8192)],
              Attn(8, 16, 2048), act="student_t", attn_dist="student_t"),
    5: Config(5, "8B-scale block: hidden 4096, 32 heads, MLP 14336 gated, 2x4096 tokens",
              [Linear("qkv", 8192, 12288, 4096), Linear("out", 8192, 4096, 4096),
               Linear("gate", 8192, 14336, 4096), Linear("up", 8192, 14336, 4096),
               Linear("down", 8192, 4096, 14336)],
              Attn(2, 32, 4096), outlier_cols=2, outlier_factor=1000.0),
}


def _rng(cid, stream):
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([BASE_SEED + cid, stream])))


def linear_tensors(cfg, idx, want=("X", "W", "dY")):
    """bf16 bit patterns (uint16 arrays) of layer `idx` of `cfg`: X [M,K], W [N,K], dY [M,N]."""
    lin = cfg.linears[idx]
    out = {}
    if "X" in want:
        rng = _rng(cfg.cid, 10 * idx + 0)
        if cfg.act == "student_t":
            x = student_t(rng, (lin.M, lin.K), 3.0)
        else:
            x = normal(rng, (lin.M, lin.K))
        if cfg.outlier_cols:
            scale_columns(x, rng, cfg.outlier_cols, cfg.outlier_factor)
        out["X"] = f32_to_bf16_bits(x)
    if "W" in want:
        out["W"] = f32_to_bf16_bits(normal(_rng(cfg.cid, 10 * idx + 1), (lin.N, lin.K), 0.02))
    if "dY" in want:
        rng = _rng(cfg.cid, 10 * idx + 2)
        if cfg.act == "student_t":
            g = student_t(rng, (lin.M, lin.N), 3.0, cfg.grad_std)
        else:
            g = normal(rng, (lin.M, lin.N), cfg.grad_std)
        out["dY"] = f32_to_bf16_bits(g)
    return out


def attention_tensors(cfg, want=("Q", "K", "V", "dO")):
    """bf16 bit patterns of Q, K, V, dO, each [B,H,S,D]."""
    a = cfg.attn
    shape = (a.B, a.H, a.S, a.D)
    out = {}
    for i, name in enumerate(("Q", "K", "V", "dO")):
        if name not in want:
            continue
        rng = _rng(cfg.cid, 1000 + i)
        std = cfg.do_std if name == "dO" else 1.0
        if cfg.attn_dist == "student_t":
            t = student_t(rng, shape, 3.0, std)
        else:
            t = normal(rng, shape, std)
        out[name] = f32_to_bf16_bits(t)
    return out


def small_linear(seed, M, N, K, outlier_cols=2, outlier_factor=50.0):
    """A small layer with the same recipe as config 1/2, for parity tests."""
    rng = np.random.Generator(np.random.PCG64(seed))
    x = normal(rng, (M, K))
    if outlier_cols and K >= outlier_cols:
        scale_columns(x, rng, outlier_cols, outlier_factor)
    w = normal(rng, (N, K), 0.02)
    g = normal(rng, (M, N), 1e-3)
    return f32_to_bf16_bits(x), f32_to_bf16_bits(w), f32_to_bf16_bits(g)


def small_attention(seed, B, H, S, D=128, do_std=1e-2):
    rng = np.random.Generator(np.random.PCG64(seed))
    shape = (B, H, S, D)
    return tuple(f32_to_bf16_bits(normal(rng, shape, s)) for s in (1.0, 1.0, 1.0, do_std))

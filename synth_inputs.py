"""Seeded synthetic inputs shared by the oracle-side and the HIP-side tests and the bench.

This module holds none of the method's arithmetic (no rounding rule, no threshold test, no
log encoding, no GEMM).  It only draws random numbers and places FP64 bit patterns, so that
both sides can be fed identical inputs without sharing any code of the method itself.

Every generator is a pure function of its arguments; seeds follow
    seed = 0x240309603000 + 16 * config + tensor_ordinal.
The shapes and distributions stand in for the paper's workloads (GPT-2 117M fine-tuning and
ResNet-50 training, Empirical Results section): activations ~ N(0,1), GPT-2 weights
~ N(0, 0.02^2), He-normal convolution weights, post-ReLU activations with ~50 % exact zeros.
"""
from __future__ import annotations

import numpy as np

SEED_BASE = 0x240309603000


def seed_for(config: int, ordinal: int) -> int:
    return SEED_BASE + 16 * int(config) + int(ordinal)


def rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(int(seed)))


def normal(shape, seed: int, sigma: float = 1.0) -> np.ndarray:
    out = rng(seed).standard_normal(shape, dtype=np.float64)
    if sigma != 1.0:
        out *= sigma
    return out


# ----------------------------------------------------------------------------------------
# Workload operands
# ----------------------------------------------------------------------------------------

def tiny_gemm(config: int = 1):
    """Config 1: A, B 256x256 ~ N(0,1)."""
    return normal((256, 256), seed_for(config, 0)), normal((256, 256), seed_for(config, 1))


def gpt2_mlp_up(config: int = 2, rows: int = 8192):
    """Config 2: X rows x 768 ~ N(0,1); W 768 x 3072 ~ N(0, 0.02^2); bias zeros (GPT-2 init)."""
    X = normal((rows, 768), seed_for(config, 0))
    W = normal((768, 3072), seed_for(config, 1), 0.02)
    return X, W, np.zeros(3072, np.float64)


def post_relu(shape, seed: int) -> np.ndarray:
    """max(0, N(0,1)): the value structure of a ResNet activation feeding a convolution."""
    return np.maximum(normal(shape, seed), 0.0)


def he_normal(shape, fan_in: int, seed: int) -> np.ndarray:
    return normal(shape, seed, float(np.sqrt(2.0 / fan_in)))


# ----------------------------------------------------------------------------------------
# Bit-level placement helpers (pure integer manipulation of IEEE bit patterns)
# ----------------------------------------------------------------------------------------

def f64_from_bits(bits) -> np.ndarray:
    return np.asarray(bits, dtype=np.uint64).view(np.float64)


def bits_from_f64(x) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.float64).view(np.uint64)


def step_magnitude(x: np.ndarray, steps: np.ndarray) -> np.ndarray:
    """Move each value `steps` FP64 neighbours away from zero (negative: toward zero).
    Caller keeps |steps| far below the magnitude bits so no value crosses zero."""
    b = bits_from_f64(x).astype(np.int64) + np.asarray(steps, dtype=np.int64)
    return b.view(np.float64)


def fp32_midpoint_above(f32_values: np.ndarray) -> np.ndarray:
    """For FP32 values (given as float32), the FP64 number halfway to the next FP32 value of
    larger magnitude.  An FP32 value widened to FP64 has 29 zero low mantissa bits; the
    halfway point sets bit 28."""
    wide = np.asarray(f32_values, dtype=np.float32).astype(np.float64)
    return (bits_from_f64(wide) | np.uint64(1 << 28)).view(np.float64)


def planted_vector(n: int, seed: int, thr: int, planted_frac: float = 0.10,
                   near_miss_frac: float = 2.0 ** -10, sigma: float = 1.0):
    """Config 5 recipe.  (1 - planted_frac) of the elements ~ N(0, sigma^2); planted_frac sit at
    midpoint +- j FP64 steps with j uniform in [0, thr-1] (must be logged); near_miss_frac sit at
    j = thr or thr + 1 (must not be logged).  Returns (x, kind) with kind 0 = random,
    1 = planted inside the band, 2 = near miss."""
    g = rng(seed)
    x = g.standard_normal(n, dtype=np.float64)
    if sigma != 1.0:
        x *= sigma
    kind = np.zeros(n, np.uint8)
    u = g.random(n)
    planted = u < planted_frac
    miss = (u >= planted_frac) & (u < planted_frac + near_miss_frac)
    sel = planted | miss
    m = int(sel.sum())
    if m:
        base = g.standard_normal(m).astype(np.float32)
        base[base == 0] = np.float32(1.0)
        mid = fp32_midpoint_above(base)
        j = np.where(planted[sel], g.integers(0, max(int(thr), 1), m),
                     int(thr) + g.integers(0, 2, m)).astype(np.int64)
        side = np.where(g.random(m) < 0.5, -1, 1).astype(np.int64)
        x[sel] = step_magnitude(mid, side * j)
        kind[planted] = 1
        kind[miss] = 2
    return x, kind


def perturb_steps(x: np.ndarray, seed: int, thr: int) -> np.ndarray:
    """Auditor stand-in: every finite non-zero value moved by a seeded integer number of FP64
    steps drawn uniformly from (-thr, thr)."""
    g = rng(seed)
    x = np.ascontiguousarray(x, dtype=np.float64)
    if thr <= 1:
        return x.copy()
    s = g.integers(-(int(thr) - 1), int(thr), x.size).astype(np.int64).reshape(x.shape)
    ok = np.isfinite(x) & (np.abs(x) > 1e-300)
    return np.where(ok, step_magnitude(x, np.where(ok, s, 0)), x)


def planted_midpoint_gemm(M: int, N: int, K: int, seed: int, noise: float = 1.0):
    """Operands whose product lands on, or a few FP64 steps from, FP32 midpoints, so that two
    accumulation orders round to different sides for a large share of the outputs.
    A = [u | E] (M x K), B = [v ; F] (K x N): u_i = 2^k_i, v_j = (2 m_j + 1) 2^-24 with m_j a
    24-bit integer with its top bit set, so u_i v_j is exactly halfway between two FP32 values;
    E F is a noise term of a few FP64 steps of that product."""
    g = rng(seed)
    k_i = g.integers(-2, 3, M)
    u = np.ldexp(1.0, k_i)
    m_j = g.integers(1 << 23, 1 << 24, N).astype(np.float64)
    v = (2.0 * m_j + 1.0) * 2.0 ** -24
    scale = noise * 2.0 ** -25 / float(max(K - 1, 1)) ** 0.25
    E = g.standard_normal((M, K - 1)) * (u[:, None] * scale)
    F = g.standard_normal((K - 1, N)) * scale
    A = np.concatenate([u[:, None], E], axis=1)
    B = np.concatenate([v[None, :], F], axis=0)
    return np.ascontiguousarray(A), np.ascontiguousarray(B)


def edge_values() -> np.ndarray:
    """Hand-built FP64 values around FP32 rounding boundaries, binade edges, the subnormal
    range, overflow, zeros, infinities and NaNs (both signs)."""
    f32 = np.array([1.0, 1.0 + 2.0 ** -23, 2.0 - 2.0 ** -23, 2.0, 0.5, 3.0, 1e-3, 7.25e10,
                    2.0 ** -126, 2.0 ** -126 * (1 + 2.0 ** -23), 2.0 ** -127, 2.0 ** -149,
                    3 * 2.0 ** -149, 2.0 ** -140, 2.0 ** 127, np.finfo(np.float32).max,
                    2.0 ** 100, 2.0 ** -100], dtype=np.float32)
    vals = []
    wide = bits_from_f64(f32.astype(np.float64)).astype(np.int64)
    for b in wide:
        for centre in (b, b + (1 << 28), b - (1 << 28), b + (1 << 29)):
            vals.append(centre + np.arange(-64, 65, dtype=np.int64))
    bits = np.concatenate(vals)
    specials = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 5e-324, 2.0 ** -1074 * 3, 2.0 ** -1022,
                         2.0 ** -150, 2.0 ** -151, 2.0 ** -150 * (1 + 2.0 ** -52),
                         2.0 ** -150 * (1 - 2.0 ** -53), 2.0 ** -149 * 1.5, 2.0 ** -149 * 2.5,
                         2.0 ** 128, 2.0 ** 128 * (1 + 2.0 ** -24), 2.0 ** 128 * (1 + 2.0 ** -24 + 2.0 ** -52),
                         2.0 ** 128 - 2.0 ** 103, 2.0 ** 128 - 2.0 ** 103 - 2.0 ** 75,
                         2.0 ** 128 - 2.0 ** 103 + 2.0 ** 75, 2.0 ** 200, 1.7976931348623157e308],
                        dtype=np.float64)
    pos = np.concatenate([bits.view(np.float64), specials])
    nan_payload = np.array([0x7FF0000000000001, 0xFFF8000000000000, 0x7FFFFFFFFFFFFFFF],
                           dtype=np.uint64).view(np.float64)
    return np.concatenate([pos, -pos, nan_payload])

"""Pins for the oracle's rounding amounts b_r < 32: rnd, boundary distance, ternary code, log,
rev and the threshold statistics on the grid of 32-bit floats whose last 32 - b_r mantissa bits
are zero.

Pinned against exact rational arithmetic written from the definition (tests/exact.py), against
library conversions where a b_r grid coincides with a hardware format (bfloat16 = 16, and the
FP16 bit strings the paper prints for its accumulation-order table = 19 inside FP16's normal
range), the closed form of the spacing that the threshold search uses as its upper end, and the
invariants of the method (idempotence, monotonicity, replay within the threshold band).
"""
import math
import os
import struct

import numpy as np
import pytest

import exact
import synth_inputs as si
from oracle import vt_oracle as vo

BS = [31, 30, 29, 28, 27, 26, 19, 16, 10]
HERE = os.path.dirname(os.path.abspath(__file__))


def _f32(bits):
    return struct.unpack("<f", struct.pack("<I", bits))[0]


def _values(b, seed):
    """Edge values, random bit patterns over the whole FP32 exponent range and beyond, and values
    planted on and next to the midpoints of the b-bit grid."""
    g = si.rng(seed)
    bits = g.integers(0, 1 << 64, 600, dtype=np.uint64)
    e = g.integers(1023 - 160, 1023 + 130, 600, dtype=np.uint64)
    band = ((bits & np.uint64(0x800FFFFFFFFFFFFF)) | (e << np.uint64(52))).view(np.float64)
    k = 32 - b
    base = g.standard_normal(300).astype(np.float32).view(np.uint32) & np.uint32(~((1 << k) - 1) & 0xFFFFFFFF)
    base = base.view(np.float32).astype(np.float64)
    base[base == 0] = 1.0
    mid_bits = base.view(np.uint64) + (np.uint64(1) << np.uint64(28 + k))          # midpoint above |base|
    steps = g.integers(-3, 4, 300).astype(np.int64)
    planted = (mid_bits.astype(np.int64) + steps).astype(np.uint64).view(np.float64)
    return np.concatenate([si.edge_values()[::7], band, planted, base])


@pytest.mark.parametrize("b", BS)
def test_rnd_distance_and_code_against_exact_rationals(b):
    xs = _values(b, si.seed_for(8, b))
    for x in xs:
        x = float(x)
        assert vo.rnd_bits(x, b) == exact.rnd32_bits(x, b), (x, b)
        assert vo.boundary_distance(x, b) == exact.boundary_distance(x, b), (x, b)
        for thr in (1, 5, 1 << 20, 1 << 27, 1 << 28):
            assert vo.ternary_code(x, thr, b) == exact.ternary_code(x, thr, b), (x, thr, b)


def test_b32_is_the_plain_conversion():
    xs = _values(32, si.seed_for(8, 32))
    for x in xs:
        x = float(x)
        assert vo.rnd_bits(x, 32) == vo.rnd32_bits(x) == exact.rnd32_bits(x)
        assert vo.boundary_distance(x, 32) == exact.boundary_distance(x)


def test_spacing_closed_form_used_by_the_threshold_search():
    # in [1, 2) the grid has b - 9 mantissa bits: spacing 2^(9 - b); the search's upper end is half of it
    for b in range(10, 33):
        assert exact.ulp32(exact.Fraction(1), b) == exact.Fraction(2) ** (9 - b)
        one_up = _f32(vo.rnd_bits(1.0 + 2.0 ** (9 - b), b))
        assert one_up == 1.0 + 2.0 ** (9 - b)                                 # a grid point
        assert _f32(vo.rnd_bits(1.0 + 0.49 * 2.0 ** (9 - b), b)) == 1.0       # below the midpoint
        assert _f32(vo.rnd_bits(1.0 + 0.5 * 2.0 ** (9 - b), b)) == 1.0        # tie: even multiple
        assert _f32(vo.rnd_bits(1.0 + 1.5 * 2.0 ** (9 - b), b)) == 1.0 + 2.0 ** (10 - b)   # tie: even multiple


def test_b16_is_bfloat16_on_fp32_inputs():
    torch = pytest.importorskip("torch")
    g = si.rng(si.seed_for(8, 100))
    x32 = np.concatenate([g.standard_normal(4000).astype(np.float32),
                          (g.standard_normal(2000) * 1e30).astype(np.float32),
                          (g.standard_normal(2000) * 1e-30).astype(np.float32)])
    want = torch.from_numpy(x32).to(torch.bfloat16).to(torch.float32).numpy().view(np.uint32)
    got = np.array([vo.rnd_bits(float(v), 16) for v in x32], np.uint32)
    assert np.array_equal(got, want)


def test_b19_reproduces_the_fp16_strings_the_paper_prints():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "floating_point_a.txt")) if l[0] not in "#\n"]
    assert len(rows) == 4
    for a, b_, c, order, f32s, f16s in rows:
        bits32 = int(f32s, 2)
        r = vo.rnd_bits(float(_f32(bits32)), 19)                   # 10 mantissa bits, as FP16 keeps
        sign, e8, m23 = r >> 31, (r >> 23) & 0xFF, r & 0x7FFFFF
        assert m23 & 0x1FFF == 0 and 1 <= e8 - 127 + 15 <= 30          # on the grid, inside FP16's normal range
        f16 = (sign << 15) | ((e8 - 127 + 15) << 10) | (m23 >> 13)
        assert format(f16, "016b") == f16s, (a, b_, c, order)


@pytest.mark.parametrize("b", [31, 28, 26, 16])
def test_rounding_invariants(b):
    xs = np.sort(_values(b, si.seed_for(8, 200 + b)))
    xs = xs[np.isfinite(xs)]
    ys = np.array([_f32(vo.rnd_bits(float(x), b)) for x in xs], np.float64)
    assert np.all(np.diff(ys[np.isfinite(ys)]) >= 0)                          # monotone
    k = 32 - b
    for x, y in zip(xs[::5], ys[::5]):
        if math.isfinite(y):
            assert vo.rnd_bits(float(y), b) == struct.unpack("<I", struct.pack("<f", y))[0]   # idempotent
            assert struct.unpack("<I", struct.pack("<f", y))[0] & ((1 << k) - 1) == 0        # zeros in the last bits
            assert vo.boundary_distance(float(y), b) == 1 << 28 or y == 0                     # grid points are never near a boundary


@pytest.mark.parametrize("b", [31, 29, 26, 16])
def test_log_replay_and_stats(b):
    k = 32 - b
    n = 4000
    thr = 1 << 12
    tau = thr * 2.0 ** -29
    g = si.rng(si.seed_for(8, 300 + b))
    xs = _values(b, si.seed_for(8, 301 + b))
    x = np.concatenate([xs, g.standard_normal(n)])
    # the auditor's values: within the band, i.e. fewer than thr * 2^k FP64 steps away
    s = g.integers(-(thr << k) + 1, thr << k, x.size).astype(np.int64)
    ok = np.isfinite(x) & (np.abs(x) > 1e-300)
    xa = np.where(ok, si.step_magnitude(x, np.where(ok, s, 0)), x)
    y, idx, dirw, cnt = vo.round_log(x, tau, b_r=b)
    codes = np.array([exact.ternary_code(float(v), thr, b) for v in x])
    assert np.array_equal(np.flatnonzero(codes != 1), idx) and cnt == idx.size
    assert np.array_equal(np.unpackbits(dirw.view(np.uint8), bitorder="little")[:cnt], (codes[idx] == 2).astype(np.uint8))
    assert np.array_equal(y.view(np.uint32), np.array([exact.rnd32_bits(float(v), b) for v in x], np.uint32))
    # rev against directed rounding in exact rationals, and the method's guarantee
    ya = vo.round_replay(xa, idx, dirw, b_r=b)
    want = np.array([exact.replay_bits(float(v), int(c), b) for v, c in zip(xa, codes)], np.uint32)
    assert np.array_equal(ya.view(np.uint32), want)
    same_binade = np.frexp(x)[1] == np.frexp(xa)[1]
    assert np.array_equal(ya.view(np.uint32)[ok & same_binade], y.view(np.uint32)[ok & same_binade])
    # packed ternary form carries the same codes and replays to the same values
    yd, tlog, cd = vo.round_log_dense(x, tau, b_r=b)
    assert cd == cnt and np.array_equal(yd.view(np.uint32), y.view(np.uint32))
    assert np.array_equal(vo.round_replay_dense(xa, tlog, b_r=b).view(np.uint32), ya.view(np.uint32))
    # statistics: flips and the smallest threshold that logs them, brute force
    st = vo.threshold_stats(x, xa, b_r=b)
    ra = np.array([exact.rnd32_bits(float(v), b) for v in xa], np.uint32)
    flip = y.view(np.uint32) != ra
    assert st["n_flip"] == int(flip.sum())
    need = [1 + max(exact.boundary_distance(float(u), b), exact.boundary_distance(float(v), b))
            for u, v in zip(x[flip], xa[flip])]
    assert st["thr_flip"] == (max(need) if need else 0)


def test_invalid_rounding_amounts_are_rejected():
    x = np.ones(4)
    for b in (9, 33, 0, -1):
        with pytest.raises(ValueError):
            vo.round_log(x, 0.1, b_r=b)
        with pytest.raises(ValueError):
            vo.threshold_stats(x, x, b_r=b)

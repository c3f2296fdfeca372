"""Pins for the CPU oracle's rounding, logging and replay (no GPU).

The oracle (oracle/vt_oracle.c) is checked against things other than itself:
  * exact rational arithmetic written from the IEEE definition and the paper's Algorithm "log"
    and primitive "rev" (tests/exact.py);
  * library routines: numpy's float64->float32 cast, the host conversion instruction under
    directed rounding modes (tests/directed_cast.c);
  * values the paper prints (tests/golden/);
  * closed forms and invariants (scale invariance, symmetry, logged fraction = 2 tau on smooth
    data, the trainer/auditor replay invariant and its tightness).
"""
import ctypes as C
import math
import os
import subprocess
import sys

import numpy as np
import pytest

import exact
import synth_inputs as si
from oracle import vt_oracle as vo

HERE = os.path.dirname(os.path.abspath(__file__))
TWO28 = 1 << 28


def _bits(y):
    return np.ascontiguousarray(y, np.float32).view(np.uint32)


@pytest.fixture(scope="module")
def edges():
    return si.edge_values()


@pytest.fixture(scope="module")
def directed():
    so = os.path.join(HERE, "_directed_cast.so")
    subprocess.check_call(["gcc", "-O1", "-frounding-math", "-shared", "-fPIC", "-o", so,
                           os.path.join(HERE, "directed_cast.c"), "-lm"])
    lib = C.CDLL(so)
    lib.cast_with_mode.argtypes = [C.POINTER(C.c_double), C.c_uint64, C.c_int, C.POINTER(C.c_float)]

    def run(x, mode):
        x = np.ascontiguousarray(x, np.float64)
        y = np.empty(x.size, np.float32)
        lib.cast_with_mode(x.ctypes.data_as(C.POINTER(C.c_double)), x.size, mode,
                           y.ctypes.data_as(C.POINTER(C.c_float)))
        return y
    return run


# ------------------------------------------------------------------------------ golden values

def test_paper_table_floating_point_a_host_arithmetic():
    """The host's IEEE arithmetic (which the other pins lean on) reproduces the bit patterns
    the paper prints for its accumulation-order example."""
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "floating_point_a.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for a, b, c, order, b32, b16 in rows:
        a, b, c = (np.float32(float(v)) for v in (a, b, c))
        s = np.float32(np.float32(a + b) + c) if order == "a+b+c" else np.float32(np.float32(a + c) + b)
        assert format(int(s.view(np.uint32)), "032b") == b32
        assert format(int(np.float16(s).view(np.uint16)), "016b") == b16


def test_paper_threshold_table_conversion():
    """tau printed as c * 2^-23 (distance from the rounded value) <-> tau_ulp = 0.5 - c; the
    search interval [0.25, 0.5] * 2^-23 maps to tau_ulp in [0, 0.25] and thr in [0, 2^27]."""
    for l in open(os.path.join(HERE, "golden", "adaptive_thresholds.txt")):
        if not l.strip() or l.startswith("#"):
            continue
        name, c, t = l.split()
        if name == "search":
            assert vo.thr_from_tau(0.5 - float(t)) == 0
            assert vo.thr_from_tau(0.5 - float(c)) == 1 << 27
            continue
        assert abs((0.5 - float(c)) - float(t)) < 1e-12
        thr = vo.thr_from_tau(float(t))
        assert thr == math.ceil(exact.Fraction(float(t)) * 2 ** 29)
        # an element exactly c*ulp away from its rounded value is NOT logged (strict >),
        # one FP64 step farther is.
        x_on = 1.0 + float(exact.Fraction(float(c)) * exact.Fraction(1, 2 ** 23))
        code_exact = exact.ternary_code(x_on, thr)
        assert vo.ternary_code(x_on, thr) == code_exact


def test_thr_from_tau():
    assert vo.thr_from_tau(0.0) == 0
    assert vo.thr_from_tau(0.5) == TWO28
    assert vo.thr_from_tau(0.25) == 1 << 27
    for e in (30, 32, 40, 60):
        assert vo.thr_from_tau(2.0 ** -e) == 1       # below FP64 resolution: exact ties only
    assert vo.thr_from_tau(2.0 ** -29) == 1
    assert vo.thr_from_tau(2.0 ** -24) == 32
    assert vo.thr_from_tau(2.0 ** -29 + 2.0 ** -60) == 2
    for bad in (-1e-9, 0.5000001, float("nan"), float("inf")):
        assert vo.thr_from_tau(bad) == 0xFFFFFFFF


# ------------------------------------------------------------------------------ rnd_32

def test_rnd32_matches_exact_rational_on_edges(edges):
    for x in edges:
        assert vo.rnd32_bits(x) == exact.rnd32_bits(float(x)), float(x).hex()


def test_rnd32_matches_numpy_cast_on_random_bit_patterns():
    g = si.rng(si.seed_for(0, 1))
    bits = g.integers(0, 1 << 64, 1 << 20, dtype=np.uint64)
    x = bits.view(np.float64)
    y, _, _, _ = vo.round_log(x, 0.0)
    with np.errstate(over="ignore", invalid="ignore"):
        ref = x.astype(np.float32)
    nan = np.isnan(x)
    assert np.array_equal(_bits(y)[~nan], _bits(ref)[~nan])
    assert np.all(_bits(y)[nan] == 0x7FC00000)
    # the FP32-relevant exponent band, where rounding actually happens
    e = g.integers(1023 - 160, 1023 + 130, 1 << 20, dtype=np.uint64)
    bits = (bits & np.uint64(0x800FFFFFFFFFFFFF)) | (e << np.uint64(52))
    x = bits.view(np.float64)
    y, _, _, _ = vo.round_log(x, 0.0)
    with np.errstate(over="ignore"):
        ref = x.astype(np.float32)
    assert np.array_equal(_bits(y), _bits(ref))


def test_rnd32_ties_go_to_even():
    for f in (1.0, 1.0 + 2.0 ** -23, 1.5, 2.0 - 2.0 ** -23):
        mid = float(si.fp32_midpoint_above(np.array([f], np.float32))[0])
        lo, hi = np.float32(f), np.nextafter(np.float32(f), np.float32(4))
        expect = lo if (int(lo.view(np.uint32)) & 1) == 0 else hi
        assert vo.rnd32_bits(mid) == int(expect.view(np.uint32))
        assert vo.rnd32_bits(np.nextafter(mid, 4.0)) == int(hi.view(np.uint32))
        assert vo.rnd32_bits(np.nextafter(mid, 0.0)) == int(lo.view(np.uint32))


# ------------------------------------------------------------------------------ D, direction, log

def test_boundary_distance_and_code_match_exact_on_edges(edges):
    thrs = (0, 1, 2, 32, 1 << 20, 1 << 27, (1 << 27) + 1, TWO28 - 1, TWO28)
    for x in edges:
        x = float(x)
        assert vo.boundary_distance(x) == exact.boundary_distance(x), x.hex()
        for thr in thrs:
            assert vo.ternary_code(x, thr) == exact.ternary_code(x, thr), (x.hex(), thr)


def test_boundary_distance_invariants():
    g = si.rng(si.seed_for(0, 2))
    x = g.standard_normal(4000)
    for v in x:
        d = vo.boundary_distance(v)
        assert 0 <= d <= TWO28
        assert d == vo.boundary_distance(-v)                      # symmetry
        for k in (-100, -7, 3, 60, 140, 300):                     # scale invariance, also past FLT_MAX
            assert d == vo.boundary_distance(math.ldexp(v, k)), (v, k)
        assert (d == TWO28) == (float(np.float32(v)) == v)         # D = 2^28  <=>  x is an FP32 value
    f = g.standard_normal(200).astype(np.float32)
    assert all(vo.boundary_distance(float(v)) == TWO28 for v in f)
    mids = si.fp32_midpoint_above(f)
    assert all(vo.boundary_distance(float(m)) == 0 for m in mids)  # D = 0 <=> exact tie
    for j in (1, 5, 31, 1000):
        assert all(vo.boundary_distance(float(m)) == j for m in si.step_magnitude(mids, np.full(200, j)))
        assert all(vo.boundary_distance(float(m)) == j for m in si.step_magnitude(mids, np.full(200, -j)))


def test_direction_is_by_value_for_both_signs():
    mid = float(si.fp32_midpoint_above(np.array([1.25], np.float32))[0])
    above, below = np.nextafter(mid, 2.0), np.nextafter(mid, 1.0)
    assert vo.ternary_code(above, 8) == 2          # rounds up to the larger float
    assert vo.ternary_code(below, 8) == 0
    assert vo.ternary_code(-above, 8) == 0         # -x rounds to the more negative float: down
    assert vo.ternary_code(-below, 8) == 2
    assert vo.ternary_code(above, 1) == 1          # one step off the tie is outside thr = 1
    assert vo.ternary_code(mid, 1) in (0, 2)


def test_round_log_matches_exact_on_edges_and_respects_cap(edges):
    for thr_tau in (2.0 ** -24, 0.25, 0.5, 0.0):
        thr = vo.thr_from_tau(thr_tau)
        y, idx, dirw, count = vo.round_log(edges, thr_tau)
        codes = [exact.ternary_code(float(v), thr) for v in edges]
        want_idx = [i for i, c in enumerate(codes) if c != 1]
        assert count == len(want_idx)
        assert idx.tolist() == want_idx
        for p, i in enumerate(want_idx):
            assert ((int(dirw[p >> 5]) >> (p & 31)) & 1) == (1 if codes[i] == 2 else 0)
        assert [int(b) for b in _bits(y)] == [exact.rnd32_bits(float(v)) for v in edges]
        if count > 10:
            cap = count // 3
            y2, idx2, dir2, count2 = vo.round_log(edges, thr_tau, cap=cap)
            assert count2 == count and np.array_equal(idx2, idx[:cap]) and np.array_equal(_bits(y2), _bits(y))
            full = cap // 32
            assert np.array_equal(dir2[:full], dirw[:full])
            if cap % 32:
                m = (1 << (cap % 32)) - 1
                assert int(dir2[full]) == int(dirw[full]) & m


def test_logged_fraction_closed_form():
    """On smooth data the position inside an FP32 cell is uniform, so P(logged) = 2 tau_ulp."""
    x = si.normal(1 << 20, si.seed_for(0, 3))
    for tau in (2.0 ** -4, 0.25, 2.0 ** -8):
        _, _, _, count = vo.round_log(x, tau)
        p = 2 * tau
        sd = math.sqrt(p * (1 - p) / x.size)
        assert abs(count / x.size - p) < 5 * sd
    _, _, _, count = vo.round_log(x, 0.5)
    assert count == x.size - int(np.sum(x.astype(np.float32).astype(np.float64) == x))


def test_thr_one_logs_exactly_the_planted_ties():
    x, kind = si.planted_vector(1 << 16, si.seed_for(5, 0), thr=1)
    y, idx, dirw, count = vo.round_log(x, 2.0 ** -40)
    planted = np.flatnonzero(kind == 1)
    assert count == planted.size and np.array_equal(idx, planted.astype(np.uint32))
    # exact ties go to the even neighbour: direction bit = 1 iff that neighbour is above x
    for p, i in enumerate(idx[:2000]):
        assert ((int(dirw[p >> 5]) >> (p & 31)) & 1) == int(float(y[i]) > x[i])
        assert int(_bits(y[i:i + 1])[0]) & 1 == 0


def test_planted_band_and_near_misses():
    thr = 32
    x, kind = si.planted_vector(1 << 16, si.seed_for(5, 1), thr=thr)
    _, idx, _, count = vo.round_log(x, 2.0 ** -24)
    logged = np.zeros(x.size, bool)
    logged[idx] = True
    assert logged[kind == 1].all()
    assert not logged[kind == 2].any()
    assert (kind == 2).sum() > 20


# ------------------------------------------------------------------------------ replay

def test_replay_matches_exact_directed_rounding_on_edges(edges):
    n = edges.size
    idx = np.arange(n, dtype=np.uint32)
    for bit in (0, 1):
        dirw = np.full((n + 31) // 32, 0xFFFFFFFF if bit else 0, np.uint32)
        y = vo.round_replay(edges, idx, dirw)
        want = [exact.replay_bits(float(v), 2 if bit else 0) for v in edges]
        assert [int(b) for b in _bits(y)] == want
    y = vo.round_replay(edges, idx[:0], np.zeros(1, np.uint32), count=0)
    assert [int(b) for b in _bits(y)] == [exact.rnd32_bits(float(v)) for v in edges]


def test_replay_matches_host_directed_conversion(directed, edges):
    """Library pin: rev with direction d equals the host's own conversion under
    FE_DOWNWARD / FE_UPWARD; with no log entry it equals FE_TONEAREST."""
    g = si.rng(si.seed_for(0, 4))
    bits = g.integers(0, 1 << 64, 1 << 18, dtype=np.uint64)
    e = g.integers(1023 - 160, 1023 + 130, bits.size, dtype=np.uint64)
    x = np.concatenate([((bits & np.uint64(0x800FFFFFFFFFFFFF)) | (e << np.uint64(52))).view(np.float64),
                        edges[~np.isnan(edges)]])
    n = x.size
    idx = np.arange(n, dtype=np.uint32)
    for mode, word in ((1, 0), (2, 0xFFFFFFFF)):
        y = vo.round_replay(x, idx, np.full((n + 31) // 32, word, np.uint32))
        assert np.array_equal(_bits(y), _bits(directed(x, mode)))
    y = vo.round_replay(x, idx[:0], np.zeros(1, np.uint32), count=0)
    assert np.array_equal(_bits(y), _bits(directed(x, 0)))


def test_replay_uses_entry_p_for_element_idx_p():
    x = si.fp32_midpoint_above(np.array([1.0, 1.5, 1.75, 3.0, 5.0], np.float32))
    x = si.step_magnitude(x, np.array([3, -3, 3, -3, 3]))
    idx = np.array([1, 2, 4], np.uint32)
    dirw = np.array([0b101], np.uint32)            # entry0 (elem 1): up, entry1 (elem 2): down, entry2 (elem 4): up
    y = vo.round_replay(x, idx, dirw)
    want = [exact.rnd32_bits(x[0]), exact.round_directed_bits(x[1], True), exact.round_directed_bits(x[2], False),
            exact.rnd32_bits(x[3]), exact.round_directed_bits(x[4], True)]
    assert [int(b) for b in _bits(y)] == want
    assert int(_bits(y)[1]) != exact.rnd32_bits(x[1])      # element 1 really was corrected
    assert int(_bits(y)[2]) != exact.rnd32_bits(x[2])


# ------------------------------------------------------------------------------ the invariant

@pytest.mark.parametrize("centre", [1.0, 1.9999998807907104, 2.0, 0.75, -1.25, 2.0 ** -126, 3.0e38])
@pytest.mark.parametrize("thr", [1, 4, 32])
def test_trainer_auditor_invariant_and_tightness(centre, thr):
    """If the auditor's FP64 value is fewer than thr FP64 steps from the trainer's, replaying
    the trainer's log reproduces the trainer's FP32 value bit for bit; at exactly thr steps a
    counter-example exists.  Brute force around an FP32 value, its midpoints and a binade edge."""
    f = np.float32(centre)
    wide = int(si.bits_from_f64(np.array([f], np.float64)).view(np.int64)[0])
    counter = 0
    for c in (wide, wide + (1 << 28), wide - (1 << 28)):
        xt = (np.arange(-3 * thr - 2, 3 * thr + 3, dtype=np.int64) + c).view(np.float64)
        yT, idx, dirw, count = vo.round_log(xt, thr * 2.0 ** -29)
        for delta in range(-thr, thr + 1):
            xa = si.step_magnitude(xt, np.full(xt.size, delta))
            yA = vo.round_replay(xa, idx, dirw)
            same = _bits(yA) == _bits(yT)
            if abs(delta) < thr:
                assert same.all(), (centre, thr, delta)
            else:
                counter += int((~same).sum())
    assert counter > 0


def test_invariant_on_perturbed_planted_vector():
    for thr, tau in ((1, 2.0 ** -40), (32, 2.0 ** -24), (1 << 20, 2.0 ** -9)):
        x, _ = si.planted_vector(1 << 16, si.seed_for(5, 2), thr=thr)
        xa = si.perturb_steps(x, si.seed_for(5, 3), thr)
        yT, idx, dirw, _ = vo.round_log(x, tau)
        yA = vo.round_replay(xa, idx, dirw)
        assert np.array_equal(_bits(yA), _bits(yT))
        if thr > 1:   # without the log the auditor does diverge: the test is not vacuous
            plain = vo.round_replay(xa, idx[:0], np.zeros(1, np.uint32), count=0)
            assert (_bits(plain) != _bits(yT)).sum() > 0

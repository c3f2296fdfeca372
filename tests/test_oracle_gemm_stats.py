"""Pins for the CPU oracle's GEMM and threshold statistics (no GPU).

GEMM: exact rational dot products on tiny random problems (error bound K 2^-53 sum|a||b|),
small-integer matrices where every summation order must be exactly right, transposed operands,
alpha and bias placement, numpy's matmul as a library cross-check.
Statistics: brute force in Python integers; Algorithm "threshold" (collection + binary search,
oracle/threshold_search.py, exact rationals) against the closed form thr_flip.
"""
from fractions import Fraction
import math

import numpy as np
import pytest

import exact
import synth_inputs as si
from oracle import vt_oracle as vo
from oracle import threshold_search as ts


def _exact_gemm(A, B, alpha, bias):
    M, K = A.shape
    N = B.shape[1]
    out = [[Fraction(float(alpha)) * exact.exact_dot(A[i, :], B[:, j]) + (Fraction(float(bias[j])) if bias is not None else 0)
            for j in range(N)] for i in range(M)]
    return out


@pytest.mark.parametrize("order", [0, 1, 2])
@pytest.mark.parametrize("shape", [(3, 5, 7), (8, 8, 8), (1, 1, 1), (4, 2, 13)])
def test_gemm_against_exact_rationals(order, shape):
    M, N, K = shape
    g = si.rng(si.seed_for(1, 8) + M * 100 + N * 10 + K)
    A, B = g.standard_normal((M, K)), g.standard_normal((K, N))
    bias = g.standard_normal(N)
    alpha = 0.125 if order != 1 else -1.7
    C = vo.gemm_f64(A, B, alpha=alpha, bias=bias, order=order)
    E = _exact_gemm(A, B, alpha, bias)
    for i in range(M):
        for j in range(N):
            bound = (K + 2) * 2.0 ** -53 * (abs(alpha) * float(np.abs(A[i]) @ np.abs(B[:, j])) + abs(bias[j]))
            err = abs(Fraction(float(C[i, j])) - E[i][j])
            assert err <= Fraction(bound), (i, j, float(err), bound)
            if order == 2:      # extended accumulation: within one rounding of the exact value
                assert err <= Fraction(2.0 ** -52 * max(abs(float(E[i][j])), 1e-300)) + Fraction(2.0 ** -62 * bound)


def test_gemm_small_integers_every_order_is_exact():
    g = si.rng(si.seed_for(1, 9))
    A = g.integers(-50, 51, (17, 33)).astype(np.float64)
    B = g.integers(-50, 51, (33, 9)).astype(np.float64)
    bias = g.integers(-9, 10, 9).astype(np.float64)
    want = 2.0 * (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float64) + bias
    for order in (0, 1, 2):
        assert np.array_equal(vo.gemm_f64(A, B, alpha=2.0, bias=bias, order=order), want)


def test_gemm_transposed_operands_and_orders():
    g = si.rng(si.seed_for(1, 10))
    A, B = g.standard_normal((6, 11)), g.standard_normal((11, 5))
    C0 = vo.gemm_f64(A, B, order=0)
    assert np.array_equal(vo.gemm_f64(np.ascontiguousarray(A.T), B, transA=True, order=0), C0)
    assert np.array_equal(vo.gemm_f64(A, np.ascontiguousarray(B.T), transB=True, order=0), C0)
    assert np.array_equal(vo.gemm_f64(np.ascontiguousarray(A.T), np.ascontiguousarray(B.T),
                                      transA=True, transB=True, order=0), C0)
    # forward order is literally the left-to-right sum; reversed order is the right-to-left sum
    for i in range(6):
        for j in range(5):
            acc = 0.0
            for k in range(11):
                acc = acc + A[i, k] * B[k, j]
            assert C0[i, j] == acc
    C1 = vo.gemm_f64(A, B, order=1)
    assert np.array_equal(C1, vo.gemm_f64(A[:, ::-1].copy(), B[::-1, :].copy(), order=0))
    assert np.allclose(C0, A @ B, rtol=0, atol=1e-13)


def test_gemm_orders_do_diverge_on_larger_problem():
    A, B = si.tiny_gemm()
    C0 = vo.gemm_f64(A[:32], B, order=0)
    C1 = vo.gemm_f64(A[:32], B, order=1)
    C2 = vo.gemm_f64(A[:32], B, order=2)
    assert (C0 != C1).mean() > 0.5                 # accumulation order changes low bits
    norm = np.linalg.norm(A[:32], axis=1)[:, None] * np.linalg.norm(B, axis=0)[None, :]
    assert np.max(np.abs(C0 - C2) / norm) < 1e-14
    assert np.max(np.abs(C1 - C2) / norm) < 1e-14
    assert np.max(np.abs(A[:32] @ B - C2) / norm) < 1e-14


# --------------------------------------------------------------------------------- statistics

def _brute_stats(y1, y2):
    n_flip, thr_flip, mx = 0, 0, 0
    hist = [0] * 65
    for a, b in zip(y1, y2):
        d = abs(exact.ord64(float(a)) - exact.ord64(float(b)))
        hist[d.bit_length()] += 1
        mx = max(mx, d)
        if exact.rnd32_bits(float(a)) != exact.rnd32_bits(float(b)):
            n_flip += 1
            thr_flip = max(thr_flip, 1 + max(exact.boundary_distance(float(a)), exact.boundary_distance(float(b))))
    return n_flip, thr_flip, mx, hist


def test_threshold_stats_brute_force():
    thr = 64
    x, _ = si.planted_vector(6000, si.seed_for(6, 0), thr=thr, planted_frac=0.3)
    y2 = si.perturb_steps(x, si.seed_for(6, 1), thr)
    x[:4] = [0.0, -0.0, 1.0, -1.0]
    y2[:4] = [-0.0, 0.0, -1.0, 1.0]                 # sign flips: huge ordinal distances
    s = vo.threshold_stats(x, y2)
    n_flip, thr_flip, mx, hist = _brute_stats(x, y2)
    assert s["n_flip"] == n_flip and n_flip > 50
    assert s["thr_flip"] == thr_flip and 0 < thr_flip
    assert s["max_ulp64_diff"] == mx
    assert s["hist"].tolist() == hist
    assert int(s["hist"].sum()) == x.size


def test_threshold_stats_identical_inputs_and_symmetry():
    x = si.normal(5000, si.seed_for(6, 2))
    s = vo.threshold_stats(x, x)
    assert s["n_flip"] == 0 and s["thr_flip"] == 0 and s["max_ulp64_diff"] == 0
    assert int(s["hist"][0]) == x.size
    y = si.perturb_steps(x, si.seed_for(6, 3), 1 << 27)
    a, b = vo.threshold_stats(x, y), vo.threshold_stats(y, x)
    assert a["n_flip"] == b["n_flip"] and a["thr_flip"] == b["thr_flip"]
    assert np.array_equal(a["hist"], b["hist"])


def test_thr_flip_is_the_smallest_safe_threshold():
    """Logging with thr = thr_flip makes the replay of y1's log on y2 reproduce rnd(y1)
    wherever the two roundings differed; thr_flip - 1 leaves at least one mismatch."""
    thr = 200
    x, _ = si.planted_vector(20000, si.seed_for(6, 4), thr=thr, planted_frac=0.3)
    y2 = si.perturb_steps(x, si.seed_for(6, 5), thr)
    s = vo.threshold_stats(x, y2)
    t = s["thr_flip"]
    assert 1 < t <= thr + 1 + thr
    for use, expect_clean in ((t, True), (t - 1, False)):
        yT, idx, dirw, _ = vo.round_log(x, use * 2.0 ** -29)
        yA = vo.round_replay(y2, idx, dirw)
        # and the other way round (the statistic is symmetric)
        yT2, idx2, dirw2, _ = vo.round_log(y2, use * 2.0 ** -29)
        yA2 = vo.round_replay(x, idx2, dirw2)
        clean = np.array_equal(yA.view(np.uint32), yT.view(np.uint32)) and \
            np.array_equal(yA2.view(np.uint32), yT2.view(np.uint32))
        assert clean == expect_clean


def test_algorithm_threshold_search_agrees_with_closed_form():
    """The printed binary search converges (from inside its interval) to the largest tau for
    which every collected distance is still logged: min p/exp.  In boundary units that is
    0.5 - (thr_flip - 1) 2^-29, i.e. thr_flip = 1 + max D over the flips."""
    thr = 1 << 22
    x, _ = si.planted_vector(3000, si.seed_for(6, 6), thr=thr, planted_frac=0.5)
    y2 = si.perturb_steps(x, si.seed_for(6, 7), thr)
    P = ts.collect(x, y2)
    s = vo.threshold_stats(x, y2)
    assert len(P) == 2 * s["n_flip"] and s["n_flip"] > 10
    tau_closed = ts.largest_safe_tau(P)
    eps = Fraction(1, 2 ** 23)
    # closed form in the oracle's integer unit
    assert (Fraction(1, 2) - tau_closed / eps) * 2 ** 29 == s["thr_flip"] - 1
    tau_search = ts.binary_search(P, b_r=32, T=80)
    assert Fraction(1, 4) * eps <= tau_search <= Fraction(1, 2) * eps
    assert abs(tau_search - tau_closed) < eps * Fraction(1, 2 ** 60)
    # (as printed, the value returned is the last midpoint tried, which may lie a hair above the
    # closed form; thr_flip is derived from the closed form, not from the returned value)


def test_search_interval_printed_in_the_paper():
    # upper end 0.5 * 2^(9 - b_r) is half an FP32 ulp of [1,2) at b_r = 32
    assert Fraction(1, 2) * Fraction(2) ** (9 - 32) == Fraction(1, 2 ** 24)
    assert ts.binary_search([], b_r=32, T=70) > Fraction(1, 2 ** 24) * (1 - Fraction(1, 2 ** 60))

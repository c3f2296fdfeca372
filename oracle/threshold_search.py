"""Adaptive threshold selection as the paper's Algorithm "threshold" states it, in exact
rational arithmetic.  TEST INFRASTRUCTURE ONLY (see vt_oracle.h); slow pure Python, meant for
small inputs.

The algorithm has two parts: (1) over pairs of results (y1, y2) of one layer computed on two
devices, keep |y - rnd(y)| for both members of every pair whose roundings disagree and that
sit on opposite sides of their rounded values; (2) binary-search tau between 0.25 * 2^-23 and
0.5 * 2^(9-b_r) so that every kept distance p satisfies p >= exp * tau, i.e. would be logged.

Readings taken where the printed algorithm is loose:
  - "exponent of p_i" is read as the exponent scale 2^floor(log2|y|) of the output y that the
    distance p_i belongs to (the same quantity Algorithm "log" multiplies tau by);
  - the value returned is the last midpoint tried, as printed; `largest_safe_tau` gives the
    closed form min_i p_i / exp_i that the search brackets from below.
"""
from __future__ import annotations

from fractions import Fraction
import math
import numpy as np


def _exact(v) -> Fraction:
    return Fraction(float(v))


def _exp_scale(y: float) -> Fraction:
    """2^floor(log2|y|), floored at 2^-126 where the FP32 spacing stops shrinking."""
    e = max(math.frexp(abs(y))[1] - 1, -126)
    return Fraction(2) ** e


def collect(y1, y2):
    """Part 1: list of (p, exp) for pairs whose FP32 roundings differ (Case A of the method)."""
    P = []
    for a, b in zip(np.asarray(y1, np.float64).ravel(), np.asarray(y2, np.float64).ravel()):
        if not (math.isfinite(a) and math.isfinite(b)) or a == 0.0 or b == 0.0:
            continue
        ra, rb = float(np.float32(a)), float(np.float32(b))
        if ra == rb or not (math.isfinite(ra) and math.isfinite(rb)):
            continue
        if (a > ra and b < rb) or (a < ra and b > rb):
            P.append((abs(_exact(a) - _exact(ra)), _exp_scale(a)))
            P.append((abs(_exact(b) - _exact(rb)), _exp_scale(b)))
    return P


def binary_search(P, b_r: int = 32, T: int = 60) -> Fraction:
    """Part 2, as printed: returns the last tau tried."""
    lower, upper, tau = Fraction(1, 4) * Fraction(1, 2 ** 23), Fraction(1, 2) * Fraction(2) ** (9 - b_r), Fraction(0)
    for _ in range(T):
        tau = (lower + upper) / 2
        success = True
        for p, e in P:
            if p < e * tau:
                success = False
        if success:
            lower = tau
        else:
            upper = tau
    return tau


def largest_safe_tau(P):
    """Closed form the search converges to when it lies inside the search interval."""
    return min(p / e for p, e in P) if P else None

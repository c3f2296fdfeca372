"""First-principles statements of the method in exact rational arithmetic (fractions.Fraction).

These are the pins the C oracle is held to: nothing here uses a floating-point rounding, a bit
mask or any code of the oracle or of the HIP path.  A binary64 input converts to a Fraction
exactly; FP32 is described by its value grid: multiples of ulp32 = 2^(max(E,-126)-23), finite
up to (2^24 - 1) 2^104, round-to-nearest with ties to the even multiple (IEEE 754).
"""
from __future__ import annotations

from fractions import Fraction
import math
import struct

FLT_MAX = Fraction((2 ** 24 - 1) * 2 ** 104)
TWO = Fraction(2)


def floor_log2(v: Fraction) -> int:
    """floor(log2 v) for v > 0, exact."""
    e = v.numerator.bit_length() - v.denominator.bit_length()
    if TWO ** e > v:
        e -= 1
    assert TWO ** e <= v < TWO ** (e + 1)
    return e


def ulp32(v: Fraction, b: int = 32) -> Fraction:
    """Spacing at v of the 32-bit floats whose last 32 - b mantissa bits are zero (b = 32: FP32)."""
    if v == 0:
        return TWO ** (-149 + 32 - b)
    return TWO ** (max(floor_log2(abs(v)), -126) - 23 + 32 - b)


def top_finite(b: int = 32) -> Fraction:
    """Largest finite value of that grid: b - 8 significant bits, all ones, in the top binade."""
    m = b - 9
    return Fraction((2 ** (m + 1) - 1) * 2 ** (127 - m))


def rnd32_unbounded(v: Fraction, b: int = 32) -> Fraction:
    """Nearest multiple of the spacing at v, ties to the even multiple; exponent range unbounded above."""
    u = ulp32(v, b)
    q = v / u
    lo = math.floor(q)
    frac = q - lo
    if frac > Fraction(1, 2) or (frac == Fraction(1, 2) and lo % 2 != 0):
        lo += 1
    return lo * u


def f32_bits_of_value(v: Fraction, negative_zero: bool = False) -> int:
    """Bit pattern of an exactly representable FP32 value (or +-inf given as None)."""
    f = float(v)
    if v == 0 and negative_zero:
        f = -0.0
    b = struct.pack("<f", f)
    assert Fraction(struct.unpack("<f", b)[0]) == v
    return struct.unpack("<I", b)[0]


def rnd32_bits(x: float, b: int = 32) -> int:
    """IEEE binary64 -> binary32, roundTiesToEven, as a bit pattern (b < 32: onto the coarser grid)."""
    if math.isnan(x):
        return 0x7FC00000
    if math.isinf(x):
        return 0x7F800000 if x > 0 else 0xFF800000
    v = Fraction(x)
    r = rnd32_unbounded(v, b)
    neg = math.copysign(1.0, x) < 0
    if abs(r) > FLT_MAX:
        return 0xFF800000 if neg else 0x7F800000
    return f32_bits_of_value(r, negative_zero=neg)


def round_directed_bits(x: float, up: bool, b: int = 32) -> int:
    """roundTowardPositive (up) / roundTowardNegative (not up) of a binary64 value to FP32."""
    if math.isnan(x):
        return 0x7FC00000
    if math.isinf(x):
        return 0x7F800000 if x > 0 else 0xFF800000
    v = Fraction(x)
    u = ulp32(v, b)
    q = v / u
    k = math.ceil(q) if up else math.floor(q)
    r = k * u
    neg = math.copysign(1.0, x) < 0
    top = top_finite(b)
    if r > top:
        return 0x7F800000 if up else f32_bits_of_value(top)
    if r < -top:
        return f32_bits_of_value(-top) if up else 0xFF800000
    return f32_bits_of_value(r, negative_zero=neg)


def ternary_code(x: float, thr: int, b: int = 32) -> int:
    """Algorithm "log" with tau = (1/2 - thr 2^-29) 2^-23: 2 = logged/up, 0 = logged/down,
    1 = ignore.  rnd is taken on the unbounded grid, so values that overflow FP32 are judged
    against the grid continued past FLT_MAX (the direction is still by value: rnd = +-inf)."""
    if math.isnan(x) or math.isinf(x):
        return 1
    v = Fraction(x)
    r = rnd32_unbounded(v, b)
    tau_scaled = (Fraction(1, 2) - Fraction(thr, 2 ** 29)) * ulp32(v, b)   # exp * tau
    far = abs(v - r) > tau_scaled
    if abs(r) > FLT_MAX:                       # the value actually produced is +-inf
        return 1 if not far else (2 if v > 0 else 0)
    if far and v < r:
        return 2
    if far and v > r:
        return 0
    return 1


def boundary_distance(x: float, b: int = 32) -> int:
    """floor of (ulp32/2 - |x - rnd(x)|) in units of 2^-29 ulp32; 2^28 for NaN/Inf."""
    if math.isnan(x) or math.isinf(x):
        return 1 << 28
    v = Fraction(x)
    r = rnd32_unbounded(v, b)
    u = ulp32(v, b)
    return math.floor((u / 2 - abs(v - r)) / (u / 2 ** 29))


def replay_bits(x: float, code: int, b: int = 32) -> int:
    """Primitive "rev": code 0 -> the FP32 value below x when rnd(x) went above it, code 2 ->
    the one above x when rnd(x) went below; otherwise rnd(x).  Since rnd(x) is one of the two
    FP32 neighbours of x this is roundTowardNegative / roundTowardPositive."""
    if code == 1:
        return rnd32_bits(x, b)
    return round_directed_bits(x, up=(code == 2), b=b)


def exact_dot(a, b) -> Fraction:
    return sum((Fraction(float(p)) * Fraction(float(q)) for p, q in zip(a, b)), Fraction(0))


def ord64(x: float) -> int:
    b = struct.unpack("<Q", struct.pack("<d", x))[0]
    mag = b & ((1 << 63) - 1)
    return -mag if b >> 63 else mag

"""Pins for the oracle's packed ternary log (five entries per byte).

Pinned against things other than the oracle: the radix-3 value written as a plain sum, brute force
over all 243 digit strings, the numbers the paper prints for the format (3^5 = 243 fits a byte,
8/5 = 1.6 bits per entry against log2(3) = 1.585), the per-element ternary code (itself pinned
against exact rational arithmetic elsewhere), and the sparse index/direction log, which must carry
the same decisions.
"""
import itertools
import math

import numpy as np
import pytest

import synth_inputs as si
from oracle import vt_oracle as vo


def test_format_constants_the_paper_prints():
    assert 3 ** 5 == 243 <= 256 < 3 ** 6            # five entries per byte, not six
    assert 8 / 5 == 1.6 and abs(math.log2(3) - 1.585) < 5e-4
    assert abs((1 - 1.6 / 8) - 0.80) < 1e-12        # the reduction against one byte per entry


def test_pack5_is_the_radix_3_value_for_every_digit_string():
    seen = set()
    for digits in itertools.product(range(3), repeat=5):
        b = vo.ternary_pack5(digits)
        assert b == sum(d * 3 ** j for j, d in enumerate(digits))       # element j has weight 3^j
        assert tuple(vo.ternary_unpack5(b)) == digits
        seen.add(b)
    assert seen == set(range(243))
    for b in range(243, 256):                        # not produced by the trainer: digits of b, sixth dropped
        assert tuple(vo.ternary_unpack5(b)) == tuple((b // 3 ** j) % 3 for j in range(5))


@pytest.mark.parametrize("n", [0, 1, 4, 5, 6, 9, 10, 11, 1000, 1003])
@pytest.mark.parametrize("tau", [0.0, 2.0 ** -24, 2.0 ** -6, 0.25])
def test_dense_log_carries_the_per_element_codes(n, tau):
    x, _ = si.planted_vector(n, si.seed_for(7, 1) + n, thr=max(vo.thr_from_tau(tau), 1), planted_frac=0.3)
    if n >= 10:
        x[:6] = si.edge_values()[:6]
    y, tlog, cnt = vo.round_log_dense(x, tau)
    assert tlog.size == (n + 4) // 5
    thr = vo.thr_from_tau(tau)
    codes = np.array([vo.ternary_code(float(v), thr) for v in x], np.int64)
    digits = np.array([(int(tlog[i // 5]) // 3 ** (i % 5)) % 3 for i in range(n)], np.int64)
    assert np.array_equal(digits, codes)
    for i in range(n, 5 * tlog.size):                # the tail of the last byte: ignore
        assert (int(tlog[i // 5]) // 3 ** (i % 5)) % 3 == 1
    assert cnt == int((codes != 1).sum())
    # same decisions as the sparse log, same FP32 values
    ys, idx, dirw, count = vo.round_log(x, tau)
    assert np.array_equal(y.view(np.uint32), ys.view(np.uint32)) and count == cnt
    assert np.array_equal(np.flatnonzero(codes != 1), idx)
    bits = np.unpackbits(dirw.view(np.uint8), bitorder="little")[:count]
    assert np.array_equal(bits, (codes[idx] == 2).astype(np.uint8))


@pytest.mark.parametrize("thr,tau", [(1, 2.0 ** -40), (64, 2.0 ** -23), (1 << 27, 0.25)])
def test_dense_replay_equals_sparse_replay_and_reproduces_the_trainer(thr, tau):
    n = 5003
    x, _ = si.planted_vector(n, si.seed_for(7, 2), thr=thr, planted_frac=0.3)
    xa = si.perturb_steps(x, si.seed_for(7, 3), thr)
    y, tlog, _ = vo.round_log_dense(x, tau)
    _, idx, dirw, _ = vo.round_log(x, tau)
    ya = vo.round_replay_dense(xa, tlog)
    assert np.array_equal(ya.view(np.uint32), vo.round_replay(xa, idx, dirw).view(np.uint32))
    assert np.array_equal(ya.view(np.uint32), y.view(np.uint32))            # 0 mismatches
    # an all-ignore log is plain rounding
    plain = vo.round_replay_dense(xa, np.full((n + 4) // 5, 121, np.uint8))
    assert np.array_equal(plain.view(np.uint32), vo.round_log(xa, 0.0)[0].view(np.uint32))


def test_dense_replay_directions_on_edge_values():
    x = si.edge_values()
    n = x.size
    idx = np.arange(n, dtype=np.uint32)
    for code, word in ((0, 0), (2, 0xFFFFFFFF)):
        tlog = np.full((n + 4) // 5, vo.ternary_pack5([code] * 5), np.uint8)
        want = vo.round_replay(x, idx, np.full((n + 31) // 32, word, np.uint32))
        assert np.array_equal(vo.round_replay_dense(x, tlog).view(np.uint32), want.view(np.uint32))

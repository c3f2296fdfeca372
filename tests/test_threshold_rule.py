"""The library's per-layer threshold rule (vt_thr_layer_from_stats: a host function, no GPU), held to what
the method needs from a threshold rather than to its own formula: on pairs of FP64 vectors with planted
near-boundary values and divergences of several magnitudes, the oracle writes the trainer's log at the
rule's threshold, the oracle replays it on the other vector, and every FP32 output must come out equal
(Method: the auditor reproduces the trainer's rounding; Algorithm "threshold" looks for a threshold with
that property).  Without the log the same replay differs in exactly n_flip outputs, so the test is not vacuous."""
import os

import numpy as np
import pytest

import synth_inputs as si
from oracle import vt_oracle as vo


@pytest.fixture(scope="module")
def hiplib():
    import paper_2403_09603_amd as vt
    if not os.path.exists(vt.library_path()):
        from paper_2403_09603_amd import build
        build.build_lib()
    return vt


def _bits(y):
    return np.ascontiguousarray(y, np.float32).view(np.uint32)


def test_rule_is_a_capped_power_of_two_covering_both_statistics(hiplib):
    g = si.rng(si.seed_for(7, 1))
    cases = [(0, 0), (1, 0), (0, 1), (2, 1), (3, 7), (1 << 27, 0), ((1 << 27) + 1, 5), (5, 1 << 27), (0, (1 << 64) - 1),
             ((1 << 64) - 1, 0), (1 << 26, (1 << 26) - 1), (1 << 26, 1 << 26)]
    cases += [(int(a), int(b)) for a, b in zip(g.integers(0, 1 << 28, 200), g.integers(0, 1 << 28, 200))]
    for thr_flip, max_diff in cases:
        thr = hiplib.vt_thr_layer_from_stats(thr_flip, max_diff)
        need = max(thr_flip, max_diff + 1, 1)
        assert thr & (thr - 1) == 0 and 1 <= thr <= hiplib.VT_THR_LAYER_MAX
        if need <= hiplib.VT_THR_LAYER_MAX:
            assert need <= thr < 2 * need                      # the smallest power of two that covers both
        else:
            assert thr == hiplib.VT_THR_LAYER_MAX


@pytest.mark.parametrize("spread", [1, 3, 40, 1000, 1 << 20])
def test_rule_guarantees_replay_on_the_observed_pair(hiplib, spread):
    n = 60000
    x, _ = si.planted_vector(n, si.seed_for(7, 10 + spread.bit_length()), thr=4 * spread, planted_frac=0.3)
    xa = si.perturb_steps(x, si.seed_for(7, 50 + spread.bit_length()), spread + 1)   # up to `spread` steps away
    st = vo.threshold_stats(x, xa)
    assert st["n_flip"] > 0 or spread == 1
    thr = hiplib.vt_thr_layer_from_stats(st["thr_flip"], st["max_ulp64_diff"])
    assert thr < hiplib.VT_THR_LAYER_MAX
    y, idx, dirw, count = vo.round_log(x, thr * 2.0 ** -29)
    ya = vo.round_replay(xa, idx, dirw, count)
    assert np.array_equal(_bits(ya), _bits(y))
    # not vacuous: without the log the auditor's own rounding differs exactly where the statistics count a flip
    plain = vo.round_replay(xa, idx[:0], np.zeros(1, np.uint32), count=0)
    assert int((_bits(plain) != _bits(y)).sum()) == st["n_flip"]

"""GPU parity: standalone round/log, replay and threshold statistics against the CPU oracle,
element by element through the C ABI.  Bar: bit-exact FP32 outputs, index lists, direction
bits, counts and integer statistics."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import vt_oracle as vo

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def _bits(y):
    return np.ascontiguousarray(y, np.float32).view(np.uint32)


def _dir_bits(dirw, count):
    return np.unpackbits(np.ascontiguousarray(dirw, np.uint32).view(np.uint8), bitorder="little")[:count]


def _same_log(g, o):
    yg, ig, dg, cg = g
    yo, io, do, co = o
    assert cg == co
    assert np.array_equal(_bits(yg), _bits(yo))
    assert np.array_equal(ig, io)
    assert np.array_equal(_dir_bits(dg, len(ig)), _dir_bits(do, len(io)))


TAUS = [0.0, 2.0 ** -40, 2.0 ** -24, 2.0 ** -4, 0.25, 0.5]


# misalign=False: single-pass kernel; misalign=True: bit-plane + compaction path
@pytest.mark.parametrize("misalign", [False, True])
@pytest.mark.parametrize("tau", TAUS)
def test_round_log_edge_values(G, tau, misalign):
    x = si.edge_values()
    _same_log(G.gpu_round_log(x, tau, misalign=misalign), vo.round_log(x, tau))


@pytest.mark.parametrize("misalign", [False, True])
@pytest.mark.parametrize("n", [0, 1, 2, 63, 64, 65, 127, 129, 1023, 1025, 4095, 4096, 4097, 3 * 4096 + 17,
                               16 * 4096, 100003, 70 * 4096 + 5])
def test_round_log_ragged_sizes(G, n, misalign):
    x, _ = si.planted_vector(n, si.seed_for(1, 4) + n, thr=32, planted_frac=0.2) if n else (np.zeros(0), None)
    for tau in (2.0 ** -24, 0.25):
        _same_log(G.gpu_round_log(x, tau, misalign=misalign), vo.round_log(x, tau))


def test_round_log_paths_agree_on_many_tiles(G):
    """1200 tiles of the single-pass kernel (more than one round of its scanner) with very uneven density:
    a dense planted stretch, a long run that logs nothing, then dense again."""
    n = 600 * 8192 + 77
    x, _ = si.planted_vector(n, si.seed_for(1, 6), thr=64, planted_frac=0.9)
    x[40 * 8192:430 * 8192] = 1.5                      # FP32 values: never logged
    tau = 64 * 2.0 ** -29
    o = vo.round_log(x, tau)
    for misalign in (False, True):
        for _ in range(2):
            _same_log(G.gpu_round_log(x, tau, misalign=misalign), o)


@pytest.mark.parametrize("n", [1, 1023, 1024, 1025, 512 * 1024, 700 * 1024 + 77, 1500 * 1024 - 1])
def test_round_only_at_threshold_zero(G, n):
    """tau = 0 logs nothing and takes the plain rounding stream (workgroups of 1024 values, walked in windows
    of 512 workgroups): every FP32 value against the oracle, count 0, for both rounding amounts."""
    x, _ = si.planted_vector(n, si.seed_for(1, 7) + n, thr=32, planted_frac=0.2)
    x[: min(n, 400)] = si.edge_values()[: min(n, 400)]
    for b_r in (32, 26):
        y, idx, dirw, cnt = G.gpu_round_log(x, 0.0, b_r=b_r)
        yo, io, do, co = vo.round_log(x, 0.0, b_r=b_r)
        assert cnt == co == 0 and len(idx) == 0
        assert np.array_equal(_bits(y), _bits(yo))


@pytest.mark.parametrize("tau", [2.0 ** -30, 2.0 ** -4, 0.25])
def test_round_log_config1_vector(G, tau):
    """Config 1: 2^20 values ~ N(0,1); at tau = 2^-30 (thr = 1) random data logs nothing, so the
    same vector is also run with 1 % planted exact ties."""
    x = si.normal(1 << 20, si.seed_for(1, 2))
    _same_log(G.gpu_round_log(x, tau), vo.round_log(x, tau))
    xp, kind = si.planted_vector(1 << 20, si.seed_for(1, 3), thr=1, planted_frac=0.01)
    g = G.gpu_round_log(xp, tau)
    _same_log(g, vo.round_log(xp, tau))
    if tau == 2.0 ** -30:
        assert g[3] == int((kind == 1).sum()) > 0


def test_round_log_is_deterministic_and_cap_overflow(G):
    x, _ = si.planted_vector(50000, si.seed_for(1, 5), thr=1 << 20, planted_frac=0.3)
    tau = 2.0 ** -9
    a = G.gpu_round_log(x, tau)
    b = G.gpu_round_log(x, tau)
    assert a[3] == b[3] and all(np.array_equal(p, q) for p, q in zip(a[:3], b[:3]))
    full = vo.round_log(x, tau)
    for cap, misalign in [(c, m) for c in (0, 1, 31, 32, 33, 1000, full[3] - 1, full[3]) for m in (False, True)]:
        g = G.gpu_round_log(x, tau, cap=cap, misalign=misalign)
        o = vo.round_log(x, tau, cap=cap)
        _same_log(g, o)
        assert g[3] == full[3] and len(g[1]) == min(cap, full[3])


@pytest.mark.parametrize("thr,tau", [(1, 2.0 ** -40), (32, 2.0 ** -24), (1 << 20, 2.0 ** -9), (1 << 27, 0.25)])
def test_replay_matches_oracle_and_trainer(G, thr, tau):
    n = 3 * 4096 + 123
    x, _ = si.planted_vector(n, si.seed_for(5, 4), thr=thr, planted_frac=0.25)
    xa = si.perturb_steps(x, si.seed_for(5, 5), thr)
    yT, idx, dirw, count = G.gpu_round_log(x, tau)
    yA = G.gpu_round_replay(xa, idx, dirw)
    assert np.array_equal(_bits(yA), _bits(vo.round_replay(xa, idx, dirw)))   # GPU replay == oracle replay
    assert np.array_equal(_bits(G.gpu_round_replay(xa, idx, dirw, misalign=True)), _bits(yA))
    assert np.array_equal(_bits(yA), _bits(yT))                                # auditor == trainer: 0 mismatches
    # CPU auditor replaying the GPU trainer's log
    assert np.array_equal(_bits(vo.round_replay(xa, idx, dirw)), _bits(yT))


@pytest.mark.parametrize("layout", ["even", "front", "back", "middle", "short"])
def test_replay_with_uneven_log_density(G, layout):
    """The replay kernel guesses where a tile's entries start from the average density and falls
    back to a full search when the guess is off: logs that are dense at one end, in the middle, or
    shorter than the probe window must all give the oracle's result."""
    n = 1 << 20
    g = si.rng(si.seed_for(5, 6))
    x = g.standard_normal(n)
    u = g.random(n)
    pos = np.arange(n)
    dense = {"even": np.ones(n, bool), "front": pos < n // 16, "back": pos >= n - n // 16,
             "middle": (pos > n // 2) & (pos < n // 2 + n // 32), "short": pos < 0}[layout]
    logged = (u < np.where(dense, 0.6, 0.0005)) if layout != "even" else (u < 0.1)
    idx = np.flatnonzero(logged).astype(np.uint32)
    assert (idx.size > 20000) == (layout != "short")
    dirw = g.integers(0, 1 << 32, (idx.size + 31) // 32 + 1, dtype=np.uint64).astype(np.uint32)
    want = _bits(vo.round_replay(x, idx, dirw, count=idx.size))
    assert np.array_equal(_bits(G.gpu_round_replay(x, idx, dirw, count=idx.size)), want)
    assert np.array_equal(_bits(G.gpu_round_replay(x, idx, dirw, count=idx.size, misalign=True)), want)


def test_replay_edge_values_all_logged_and_empty(G):
    x = si.edge_values()
    n = x.size
    idx = np.arange(n, dtype=np.uint32)
    for word in (0, 0xFFFFFFFF, 0xA5A5A5A5):
        dirw = np.full((n + 31) // 32, word, np.uint32)
        want = _bits(vo.round_replay(x, idx, dirw))
        assert np.array_equal(_bits(G.gpu_round_replay(x, idx, dirw)), want)
        assert np.array_equal(_bits(G.gpu_round_replay(x, idx, dirw, misalign=True)), want)
    empty = G.gpu_round_replay(x, idx[:0], np.zeros(0, np.uint32), count=0)
    assert np.array_equal(_bits(empty), _bits(vo.round_replay(x, idx[:0], np.zeros(1, np.uint32), count=0)))
    # sparse log with entries at tile borders and stray indices >= n (ignored)
    idx2 = np.array([0, 4095, 4096, 8191, n - 1, n, n + 7], np.uint32)
    dir2 = np.array([0b1010101], np.uint32)
    assert np.array_equal(_bits(G.gpu_round_replay(x, idx2, dir2)), _bits(vo.round_replay(x, idx2, dir2)))


@pytest.mark.parametrize("n", [1, 64, 4097, 70001])
def test_threshold_stats(G, n):
    thr = 4096
    x, _ = si.planted_vector(n, si.seed_for(6, 8) + n, thr=thr, planted_frac=0.3)
    y2 = si.perturb_steps(x, si.seed_for(6, 9), thr)
    if n > 8:
        x[:4] = [0.0, -0.0, 1.0, np.inf]
        y2[:4] = [-0.0, 0.0, -1.0, np.inf]
    g, o = G.gpu_stats(x, y2), vo.threshold_stats(x, y2)
    assert g["n_flip"] == o["n_flip"] and g["thr_flip"] == o["thr_flip"]
    assert g["max_ulp64_diff"] == o["max_ulp64_diff"]
    assert np.array_equal(g["hist"], o["hist"])
    assert G.gpu_stats(x, x)["n_flip"] == 0

"""GPU parity for the element-wise and row-wise layers fused with the trainer hook.

FP64 layer outputs (debug copy) against the oracle's extended-precision evaluation within a tolerance
derived from the arithmetic (a few FP64 roundings plus the accuracy of exp / tanh / erf, and for the
row-wise layers the rounding of the row statistics); residual add and ReLU exactly.  FP32 outputs and
both log formats bit-exact against the oracle's round/log of the kernel's own FP64 values.  Two
summation orders of the row statistics stand in for two GPU types: the trainer's log replayed on the
other order's values reproduces the trainer's FP32 outputs."""
import numpy as np
import pytest

import paper_2403_09603_amd as vtlib
import synth_inputs as si
from oracle import vt_oracle as vo

pytestmark = pytest.mark.gpu

ADD, RELU, GELU_TANH, GELU_ERF, NORM, SOFTMAX = range(6)
SHAPES = [(1, 1), (7, 333), (3, 8197), (200, 768), (37, 1280)]
# layer norm and softmax over rows of 64 to 2048 columns (1024 with the index-list log) are computed a row at a
# time in registers, five rows per wave, other row lengths by a statistics pass and the element-wise pass: both
# sides of every limit, row counts that leave a wave or a workgroup partly empty, odd row lengths (rows that
# start off a 16-byte boundary)
ROW_SHAPES = [(301, 64), (100, 63), (41, 2048), (9, 2049), (5, 1024), (13, 1025), (23, 512), (11, 513), (7, 127), (6, 129)]
NORM_SHAPES = SHAPES + ROW_SHAPES


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def _bits(y):
    return np.ascontiguousarray(y, np.float32).view(np.uint32)


def _dir_bits(dirw, count):
    return np.unpackbits(np.ascontiguousarray(dirw, np.uint32).view(np.uint8), bitorder="little")[:count]


def _hook(r, tau, b_r=32):
    yo, io, do, co = vo.round_log(r["y64"].ravel(), tau, b_r=b_r)
    assert r["count"] == co and np.array_equal(_bits(r["y32"].ravel()), _bits(yo))
    if "tlog" in r:
        assert np.array_equal(r["tlog"], vo.round_log_dense(r["y64"].ravel(), tau, b_r=b_r)[1])
    else:
        assert np.array_equal(r["idx"], io) and np.array_equal(_dir_bits(r["dir"], co), _dir_bits(do, co))


def _inputs(shape, seed):
    g = si.rng(si.seed_for(9, 100 + seed))
    a = (g.standard_normal(shape) * 2.0).astype(np.float32).astype(np.float64)
    b = g.standard_normal(shape).astype(np.float32).astype(np.float64)
    if a.size > 40:
        a.ravel()[:8] = [0.0, -0.0, 40.0, -40.0, 1e-30, -1e-30, 700.0, -700.0]
    return a, b, g


@pytest.mark.parametrize("dense", [False, True])
@pytest.mark.parametrize("shape", SHAPES)
def test_elementwise_layers(G, shape, dense):
    a, b, _ = _inputs(shape, shape[1])
    tau = 2.0 ** -4
    r = G.gpu_layer(ADD, a, b, tau=tau, dense=dense)
    assert np.array_equal(r["y64"], vo.elementwise(vo.EW_ADD, a, b))          # one IEEE addition: exact
    _hook(r, tau)
    r = G.gpu_layer(RELU, a, tau=tau, dense=dense)
    assert np.array_equal(r["y64"].view(np.uint64), vo.elementwise(vo.EW_RELU, a).view(np.uint64))
    _hook(r, tau)
    for op, oop in ((GELU_TANH, vo.EW_GELU_TANH), (GELU_ERF, vo.EW_GELU_ERF)):
        r = G.gpu_layer(op, a, tau=tau, dense=dense)
        truth = vo.elementwise(oop, a, exact=True)
        # 0.5 x (1 + f): a handful of roundings and the function's own error, relative to |x|
        assert np.all(np.abs(r["y64"] - truth) <= 8 * 2.0 ** -52 * np.maximum(np.abs(a), 1e-300)), op
        _hook(r, tau)


@pytest.mark.parametrize("dense", [False, True])
@pytest.mark.parametrize("shape", NORM_SHAPES)
def test_layernorm(G, shape, dense):
    a, _, g = _inputs(shape, 50 + shape[1])
    a = a + 0.25
    gamma = (g.standard_normal(shape[1]) + 1.0).astype(np.float32).astype(np.float64)
    beta = g.standard_normal(shape[1]).astype(np.float32).astype(np.float64)
    tau = 2.0 ** -4
    truth = vo.layernorm(a, gamma, beta, 1e-5, order=2)
    xhat = np.abs(vo.layernorm(a, eps=1e-5, order=2))
    cols = shape[1]
    # error of mean and 1/std: ~ sqrt(cols) roundings each, carried through (x - mean) rstd gamma + beta
    bound = 2.0 ** -52 * (8 + 4 * np.sqrt(cols)) * (xhat + 1.0) * np.abs(gamma)[None, :] + 2.0 ** -52 * np.abs(truth) + 1e-300
    res = {}
    for variant in (0, 1):
        r = G.gpu_layer(NORM, a, gamma=gamma, beta=beta, eps=1e-5, tau=tau, variant=variant, dense=dense)
        assert np.all(np.abs(r["y64"] - truth) <= bound), float(np.max(np.abs(r["y64"] - truth) / bound))
        _hook(r, tau)
        res[variant] = r
    again = G.gpu_layer(NORM, a, gamma=gamma, beta=beta, eps=1e-5, tau=tau, variant=0, dense=dense)
    assert np.array_equal(again["y64"], res[0]["y64"])                         # deterministic
    r = G.gpu_layer(NORM, a, eps=0.0, tau=tau, dense=dense)                    # no gamma, no beta
    if cols > 1:
        np.testing.assert_allclose(r["y64"], vo.layernorm(a, eps=0.0, order=2), rtol=0, atol=1e-12)


@pytest.mark.parametrize("dense", [False, True])
@pytest.mark.parametrize("shape,period", [((1, 1), 0), ((7, 333), 0), ((24, 200), 8), ((300, 100), 100), ((64, 1024), 0),
                                          ((3, 8197), 0), ((7, 127), 4), ((23, 513), 16), ((41, 2048), 0), ((44, 1024), 11)]
                         + [(sh, 0) for sh in ROW_SHAPES])
def test_softmax(G, shape, period, dense):
    a, _, _ = _inputs(shape, 70 + shape[1])
    a = np.clip(a, -50, 50)
    tau, scale = 2.0 ** -4, 0.125
    truth = vo.softmax(a, scale, period, order=2)
    cols = shape[1]
    bound = 2.0 ** -52 * (8 + 2 * np.sqrt(cols)) * truth + 1e-300
    for variant in (0, 1):
        r = G.gpu_layer(SOFTMAX, a, scale=scale, causal_period=period, tau=tau, variant=variant, dense=dense)
        assert np.all(np.abs(r["y64"] - truth) <= bound), float(np.max(np.abs(r["y64"] - truth) / np.maximum(bound, 1e-300)))
        assert np.all((r["y64"] == 0.0) == (truth == 0.0))                     # the mask
        _hook(r, tau)


@pytest.mark.parametrize("dense", [False, True])
@pytest.mark.parametrize("shape", [(2, 1), (9, 3), (700, 64), (5000, 200), (1300, 513), (40000, 64)])
def test_batchnorm(G, shape, dense):
    a, _, g = _inputs(shape, 90 + shape[1])
    a = np.clip(a, -60, 60) + 0.25
    rows, cols = shape
    gamma = (g.standard_normal(cols) + 1.0).astype(np.float32).astype(np.float64)
    beta = g.standard_normal(cols).astype(np.float32).astype(np.float64)
    tau = 2.0 ** -4
    truth = vo.batchnorm(a, gamma, beta, 1e-5, order=2)
    xhat = np.abs(vo.batchnorm(a, eps=1e-5, order=2))
    bound = 2.0 ** -52 * (8 + 4 * np.sqrt(rows)) * (xhat + 1.0) * np.abs(gamma)[None, :] + 2.0 ** -52 * np.abs(truth) + 1e-300
    for variant in (0, 1):
        r = G.gpu_layer(6, a, gamma=gamma, beta=beta, eps=1e-5, tau=tau, variant=variant, dense=dense)
        assert np.all(np.abs(r["y64"] - truth) <= bound), float(np.max(np.abs(r["y64"] - truth) / bound))
        _hook(r, tau)
        rr = G.gpu_layer(7, a, gamma=gamma, beta=beta, eps=1e-5, tau=tau, variant=variant, dense=dense)
        assert np.array_equal(rr["y64"], np.maximum(r["y64"], 0.0))              # ReLU of the same values
        _hook(rr, tau)
    again = G.gpu_layer(6, a, gamma=gamma, beta=beta, eps=1e-5, tau=tau, variant=1, dense=dense)
    assert np.array_equal(again["y64"], r["y64"])                                # deterministic


@pytest.mark.parametrize("dense", [False, True])
@pytest.mark.parametrize("op,shape,kw", [(GELU_TANH, (37, 1280), {}), (NORM, (43, 1000), dict(eps=1e-5)), (NORM, (9, 2049), dict(eps=1e-5)),
                                         (SOFTMAX, (43, 1000), dict(scale=0.125, causal_period=7)),
                                         (SOFTMAX, (3, 8197), dict(scale=0.125)), (6, (1300, 513), dict(eps=1e-5))])
def test_without_the_fp64_debug_copy(G, op, shape, kw, dense):
    """The call as the benchmarks make it (no FP64 copy of the layer's output) writes the same FP32 values and the
    same log, bit for bit, as the call with the copy, whose FP64 values the tests above hold to the oracle."""
    a, _, g = _inputs(shape, 400 + shape[1])
    a = np.clip(a, -50, 50)
    tau = 2.0 ** -5
    for b_r in (32, 26):
        full = G.gpu_layer(op, a, tau=tau, dense=dense, b_r=b_r, **kw)
        bare = G.gpu_layer(op, a, tau=tau, dense=dense, b_r=b_r, want_y64=False, **kw)
        _hook(full, tau, b_r)
        assert bare["count"] == full["count"] and np.array_equal(_bits(bare["y32"]), _bits(full["y32"]))
        for key in ("tlog", "idx", "dir"):
            if key in full:
                assert np.array_equal(bare[key], full[key]), key


@pytest.mark.parametrize("op,kw", [(NORM, dict(eps=1e-5)), (SOFTMAX, dict(scale=0.25))])
def test_rowwise_index_list_capacity(G, op, kw):
    """A log smaller than the number of entries keeps the first `cap` entries in output order and still
    counts them all (rows held in registers: the entries of a tile leave through the scanner protocol)."""
    a, _, _ = _inputs((83, 1000), 500)
    tau = 0.25
    full = G.gpu_layer(op, a, tau=tau, **kw)
    assert full["count"] > 1000
    for cap in (0, 1, 255, 256, 257, full["count"] // 2, full["count"] - 1, full["count"]):
        part = G.gpu_layer(op, a, tau=tau, cap=cap, **kw)
        stored = min(cap, full["count"])
        assert part["count"] == full["count"] and np.array_equal(_bits(part["y32"]), _bits(full["y32"]))
        assert np.array_equal(part["idx"], full["idx"][:stored])
        assert np.array_equal(_dir_bits(part["dir"], stored), _dir_bits(full["dir"], stored))


def test_two_summation_orders_and_replay(G):
    """Layer norm and softmax over long rows: the two variants differ in low bits; the threshold from
    their statistics makes the trainer's log bring the other variant back to the trainer's outputs."""
    g = si.rng(si.seed_for(9, 300))
    a = g.standard_normal((512, 3072)).astype(np.float32).astype(np.float64)
    for op, kw in ((NORM, dict(eps=1e-5)), (SOFTMAX, dict(scale=0.5)), (6, dict(eps=1e-5))):
        r0 = G.gpu_layer(op, a, tau=0.0, variant=0, **kw)
        r1 = G.gpu_layer(op, a, tau=0.0, variant=1, **kw)
        assert (r0["y64"] != r1["y64"]).mean() > 0.05
        st = G.gpu_stats(r0["y64"], r1["y64"])
        so = vo.threshold_stats(r0["y64"], r1["y64"])
        assert st["n_flip"] == so["n_flip"] and st["thr_flip"] == so["thr_flip"]
        thr = vtlib.vt_thr_layer_from_stats(st["thr_flip"], st["max_ulp64_diff"])      # the library's rule
        assert max(st["thr_flip"], st["max_ulp64_diff"] + 1) <= thr                # not capped at 1/4 ulp
        tau = thr * 2.0 ** -29
        for dense in (False, True):
            t = G.gpu_layer(op, a, tau=tau, variant=0, dense=dense, **kw)
            if dense:
                ya = G.gpu_round_replay_dense(r1["y64"].ravel(), t["tlog"])
            else:
                ya = G.gpu_round_replay(r1["y64"].ravel(), t["idx"], t["dir"])
            assert np.array_equal(_bits(ya), _bits(t["y32"].ravel()))


def test_rounding_amount_and_validation(G):
    import paper_2403_09603_amd as vt
    a, b, _ = _inputs((9, 130), 400)
    r = G.gpu_layer(GELU_TANH, a, tau=2.0 ** -4, b_r=26)
    _hook(r, 2.0 ** -4, b_r=26)
    with pytest.raises(vt.VtError):
        G.gpu_layer(ADD, a)                                                    # second addend missing
    with pytest.raises(vt.VtError):
        G.gpu_layer(8, a)                                                      # unknown layer

"""GPU parity for rounding amounts b_r < 32: every entry point against the oracle, bit-exact."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import vt_oracle as vo

pytestmark = pytest.mark.gpu

BS = [31, 29, 26, 16, 10]


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def _bits(y):
    return np.ascontiguousarray(y, np.float32).view(np.uint32)


def _dir_bits(dirw, count):
    return np.unpackbits(np.ascontiguousarray(dirw, np.uint32).view(np.uint8), bitorder="little")[:count]


def _vector(b, n, seed, thr):
    """Random values, edge values, and values planted around the midpoints of the b_r grid."""
    g = si.rng(seed)
    k = 32 - b
    x = g.standard_normal(n)
    m = n // 3
    base = g.standard_normal(m).astype(np.float32).view(np.uint32) & np.uint32(~((1 << k) - 1) & 0xFFFFFFFF)
    base = base.view(np.float32).astype(np.float64)
    base[base == 0] = 1.0
    j = g.integers(-(2 * thr << k), (2 * thr << k) + 1, m)
    x[:m] = (base.view(np.uint64).astype(np.int64) + (1 << (28 + k)) + j).astype(np.uint64).view(np.float64)
    ev = si.edge_values()
    x[m:m + min(ev.size, n - m)] = ev[:n - m]
    return x


@pytest.mark.parametrize("misalign", [False, True])
@pytest.mark.parametrize("b", BS)
def test_round_log_replay_stats(G, b, misalign):
    n, thr = 3 * 8192 + 777, 1 << 10
    tau = thr * 2.0 ** -29
    k = 32 - b
    x = _vector(b, n, si.seed_for(8, 400 + b), thr)
    y, idx, dirw, cnt = G.gpu_round_log(x, tau, misalign=misalign, b_r=b)
    yo, io, do, co = vo.round_log(x, tau, b_r=b)
    assert cnt == co and np.array_equal(_bits(y), _bits(yo)) and np.array_equal(idx, io)
    assert np.array_equal(_dir_bits(dirw, co), _dir_bits(do, co))
    assert co > n // 10
    # auditor inside the band
    g = si.rng(si.seed_for(8, 500 + b))
    s = g.integers(-(thr << k) + 1, thr << k, n).astype(np.int64)
    ok = np.isfinite(x) & (np.abs(x) > 1e-300)
    xa = np.where(ok, si.step_magnitude(x, np.where(ok, s, 0)), x)
    ya = G.gpu_round_replay(xa, idx, dirw, misalign=misalign, b_r=b)
    assert np.array_equal(_bits(ya), _bits(vo.round_replay(xa, idx, dirw, b_r=b)))
    same = ok & (np.frexp(x)[1] == np.frexp(xa)[1])
    assert np.array_equal(_bits(ya)[same], _bits(y)[same])
    # packed ternary form
    yd, tlog, cd = G.gpu_round_log_dense(x, tau, misalign=misalign, b_r=b)
    _, to, _ = vo.round_log_dense(x, tau, b_r=b)
    assert np.array_equal(tlog, to) and cd == co and np.array_equal(_bits(yd), _bits(yo))
    assert np.array_equal(_bits(G.gpu_round_replay_dense(xa, tlog, misalign=misalign, b_r=b)), _bits(ya))
    # statistics
    st, so = G.gpu_stats(x, xa, b_r=b), vo.threshold_stats(x, xa, b_r=b)
    assert st["n_flip"] == so["n_flip"] and st["thr_flip"] == so["thr_flip"]
    assert st["max_ulp64_diff"] == so["max_ulp64_diff"] and np.array_equal(st["hist"], so["hist"])


@pytest.mark.parametrize("b", [30, 26, 16])
def test_gemm_and_conv_with_a_rounding_amount(G, b):
    g = si.rng(si.seed_for(8, 600 + b))
    tau = 2.0 ** -4
    for (M, N, K, tA) in [(130, 70, 37, False), (256, 256, 64, False), (64, 147, 6000, True)]:
        A = g.standard_normal((K, M) if tA else (M, K))
        B = g.standard_normal((K, N))
        bias = g.standard_normal(N)
        for variant in (0, 1):
            r = G.gpu_gemm(A, B, transA=tA, alpha=0.5, bias=bias, tau=tau, variant=variant, b_r=b)
            r32 = G.gpu_gemm(A, B, transA=tA, alpha=0.5, bias=bias, tau=tau, variant=variant)
            assert np.array_equal(r["C64"], r32["C64"])                       # same FP64 layer, other rounding
            yo, io, do, co = vo.round_log(r["C64"].ravel(), tau, b_r=b)
            assert r["count"] == co and np.array_equal(_bits(r["C32"].ravel()), _bits(yo))
            assert np.array_equal(r["idx"], io) and np.array_equal(_dir_bits(r["dir"], co), _dir_bits(do, co))
            d = G.gpu_gemm_dense(A, B, transA=tA, alpha=0.5, bias=bias, tau=tau, variant=variant, b_r=b)
            assert np.array_equal(d["tlog"], vo.round_log_dense(r["C64"].ravel(), tau, b_r=b)[1])
    X = np.maximum(g.standard_normal((2, 12, 11, 8)), 0.0)
    Wt = g.standard_normal((3, 3, 8, 16)) * 0.1
    r = G.gpu_conv(0, X, Wt, 3, 3, pad=1, tau=tau, b_r=b)
    yo, io, do, co = vo.round_log(r["C64"].ravel(), tau, b_r=b)
    assert r["count"] == co and np.array_equal(_bits(r["C32"].ravel()), _bits(yo)) and np.array_equal(r["idx"], io)
    truth = vo.conv2d_fwd(X, Wt, pad=1, order=2).reshape(-1, 16)
    assert np.max(np.abs(r["C64"] - truth)) < 1e-12 * 9 * 8 * 4
    dY = g.standard_normal((2, 6, 6, 16))
    r = G.gpu_conv(2, dY, Wt, 3, 3, stride=2, pad=1, tau=tau, b_r=b, xshape=(2, 12, 11, 8))      # input gradient
    yo, io, do, co = vo.round_log(r["C64"].ravel(), tau, b_r=b)
    assert r["count"] == co and np.array_equal(_bits(r["C32"].ravel()), _bits(yo)) and np.array_equal(r["idx"], io)
    truth = vo.conv2d_dgrad(dY, Wt, (2, 12, 11, 8), stride=2, pad=1, order=2).reshape(-1, 8)
    assert np.max(np.abs(r["C64"] - truth)) < 1e-12 * 9 * 16 * 4


def test_padded_output_with_a_rounding_amount_is_refused(G):
    import paper_2403_09603_amd as vt
    g = si.rng(si.seed_for(8, 700))
    with pytest.raises(vt.VtError, match="unsupported"):
        G.gpu_gemm(g.standard_normal((70, 33)), g.standard_normal((33, 50)), ldc=64, b_r=26)

"""GPU parity for the packed ternary log (five entries per byte): trainer hook, replay, and the
GEMM / convolution entry points writing that format.  Bytes, FP32 outputs and counts are
bit-exact against the oracle."""
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


@pytest.mark.parametrize("misalign", [False, True])
@pytest.mark.parametrize("n", [0, 1, 4, 5, 6, 127, 639, 640, 641, 1279, 1280, 2561, 5 * 4096 + 3, (1 << 20) + 7])
def test_round_log_dense_ragged_sizes(G, n, misalign):
    thr = 1 << 20
    tau = thr * 2.0 ** -29
    x, _ = si.planted_vector(n, si.seed_for(7, 4) + n, thr=thr, planted_frac=0.3)
    if n >= 700:
        ev = si.edge_values()
        x[100:100 + min(ev.size, 500)] = ev[:500]
    y, tlog, cnt = G.gpu_round_log_dense(x, tau, misalign=misalign)
    yo, to, co = vo.round_log_dense(x, tau)
    assert np.array_equal(_bits(y), _bits(yo))
    assert np.array_equal(tlog, to)
    assert cnt == co


@pytest.mark.parametrize("tau", [0.0, 2.0 ** -40, 2.0 ** -24, 2.0 ** -6, 0.25, 0.5])
def test_round_log_dense_edge_values(G, tau):
    x = np.concatenate([si.edge_values(), si.planted_vector(3000, si.seed_for(7, 5), thr=max(vo.thr_from_tau(tau), 1))[0]])
    y, tlog, cnt = G.gpu_round_log_dense(x, tau)
    yo, to, co = vo.round_log_dense(x, tau)
    assert np.array_equal(_bits(y), _bits(yo)) and np.array_equal(tlog, to) and cnt == co


@pytest.mark.parametrize("misalign", [False, True])
@pytest.mark.parametrize("thr,tau", [(1, 2.0 ** -40), (64, 2.0 ** -23), (1 << 27, 0.25)])
def test_replay_dense_matches_oracle_and_trainer(G, thr, tau, misalign):
    n = 7 * 640 + 333
    x, _ = si.planted_vector(n, si.seed_for(7, 6), thr=thr, planted_frac=0.3)
    xa = si.perturb_steps(x, si.seed_for(7, 7), thr)
    yT, tlog, _ = G.gpu_round_log_dense(x, tau)
    yA = G.gpu_round_replay_dense(xa, tlog, misalign=misalign)
    assert np.array_equal(_bits(yA), _bits(vo.round_replay_dense(xa, tlog)))
    assert np.array_equal(_bits(yA), _bits(yT))                       # 0 mismatches
    # the sparse log of the same tensor replays to the same values
    _, idx, dirw, _ = G.gpu_round_log(x, tau)
    assert np.array_equal(_bits(G.gpu_round_replay(xa, idx, dirw)), _bits(yA))


def test_replay_dense_every_byte_value_and_edge_values(G):
    x = si.edge_values()
    n = x.size
    g = si.rng(si.seed_for(7, 8))
    for trial in range(3):
        tlog = g.integers(0, 256, (n + 4) // 5, dtype=np.uint64).astype(np.uint8)    # includes bytes above 242
        tlog[:256] = np.arange(256, dtype=np.uint8)[:min(256, tlog.size)] if tlog.size >= 256 else tlog[:256]
        assert np.array_equal(_bits(G.gpu_round_replay_dense(x, tlog)), _bits(vo.round_replay_dense(x, tlog)))
    assert G.gpu_round_replay_dense(x[:0], np.zeros(0, np.uint8)).size == 0


@pytest.mark.parametrize("case", [
    dict(M=130, N=70, K=37), dict(M=256, N=256, K=64), dict(M=300, N=64, K=5), dict(M=17, N=1000, K=64),
    dict(M=96, N=64, K=40, batch=3, transB=True), dict(M=70, N=50, K=33, ldc=64),
    dict(M=64, N=147, K=6000, transA=True),                                        # split-K path
])
def test_gemm_writes_the_packed_log(G, case):
    M, N, K = case["M"], case["N"], case["K"]
    batch, tA, tB = case.get("batch", 1), case.get("transA", False), case.get("transB", False)
    g = si.rng(si.seed_for(7, 9) + M + N + K)
    shapeA = (K, M) if tA else (M, K)
    shapeB = (N, K) if tB else (K, N)
    A = g.standard_normal((batch,) + shapeA if batch > 1 else shapeA)
    B = g.standard_normal((batch,) + shapeB if batch > 1 else shapeB)
    bias = g.standard_normal(N)
    tau = 2.0 ** -3
    for variant in (0, 1):
        r = G.gpu_gemm_dense(A, B, transA=tA, transB=tB, alpha=0.5, bias=bias, tau=tau, variant=variant,
                             ldc=case.get("ldc"))
        yo, to, co = vo.round_log_dense(r["C64"].ravel(), tau)
        assert np.array_equal(_bits(r["C32"].ravel()), _bits(yo))
        assert np.array_equal(r["tlog"], to) and r["count"] == co
        s = G.gpu_gemm(A, B, transA=tA, transB=tB, alpha=0.5, bias=bias, tau=tau, variant=variant, ldc=case.get("ldc"))
        assert np.array_equal(s["C64"], r["C64"]) and s["count"] == r["count"]       # same layer, other format

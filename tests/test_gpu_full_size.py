"""GPU parity at the full sizes and launch configurations that bench.py times.

Config 2 (GPT-2 117M MLP up-projection, 8192 x 768 x 3072): FP64 values against the oracle on sampled
rows; everything derived from them (25 M FP32 outputs, the whole log) bit-exact against the oracle's
round/log of the kernel's own FP64 values; replay by GPU and by the CPU oracle.
Config 5 (2^28 values, 10 % planted near midpoints): the oracle on sampled windows, plus properties
that hold at any size (ordering, planted band logged, near misses not, direction by value, replay
of the perturbed vector reproduces the trainer's outputs exactly)."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import vt_oracle as vo

pytestmark = pytest.mark.gpu


def _bits(y):
    return np.ascontiguousarray(y, np.float32).view(np.uint32)


def _dir_bits(dirw, count):
    return np.unpackbits(np.ascontiguousarray(dirw, np.uint32).view(np.uint8), bitorder="little")[:count]


def test_config2_full_size():
    import torch
    import paper_2403_09603_amd as vt
    dev = "cuda"
    M, K, N = 8192, 768, 3072
    X, W, bias = si.gpt2_mlp_up(config=2, rows=M)
    Xd, Wd, bd = (torch.from_numpy(a).to(dev) for a in (X, W, bias))
    total = M * N
    ws = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, M, N, K, 1))
    out = {}
    for variant in (0, 1):
        C32 = torch.empty((M, N), dtype=torch.float32, device=dev)
        C64 = torch.empty((M, N), dtype=torch.float64, device=dev)
        log = vt.alloc_log(total)
        vt.vt_gemm_f64_round_log(False, False, M, N, K, 1.0, Xd, K, 0, Wd, N, 0, bd, 1, C32, N, 0, C64, variant,
                                 0.25, log, ws)
        torch.cuda.synchronize()
        cnt = int(log.count.item())
        out[variant] = (C32.cpu().numpy().ravel(), C64.cpu().numpy().ravel(),
                        log.idx.cpu().numpy().view(np.uint32)[:cnt], log.dir.cpu().numpy().view(np.uint32)[:(cnt + 31) // 32], cnt)
    # FP64 values on sampled rows (tile borders, first, last)
    rows = [0, 1, 63, 64, 127, 128, 4095, 4096, 8191] + list(si.rng(si.seed_for(2, 7)).integers(0, M, 15))
    wn = np.linalg.norm(W, axis=0)
    for variant in (0, 1):
        c64 = out[variant][1].reshape(M, N)
        for r in rows:
            truth = vo.gemm_f64(X[r:r + 1], W, bias=bias, order=2)[0]
            assert np.all(np.abs(c64[r] - truth) <= 1e-12 * np.linalg.norm(X[r]) * wn + 1e-300)
    # everything after the FP64 value: the whole tensor, bit for bit
    for variant in (0, 1):
        c32, c64, idx, dirw, cnt = out[variant]
        yo, io, do, co = vo.round_log(c64, 0.25)
        assert cnt == co and np.array_equal(_bits(c32), _bits(yo)) and np.array_equal(idx, io)
        assert np.array_equal(_dir_bits(dirw, cnt), _dir_bits(do, co))
    # trainer = variant 0; auditors = GPU variant 1 and the CPU oracle's reversed-k rows
    c32_T, c64_T, idx, dirw, cnt = out[0]
    st = torch.zeros(68, dtype=torch.int64, device=dev)
    vt.vt_threshold_stats(torch.from_numpy(c64_T).to(dev), torch.from_numpy(out[1][1]).to(dev), st)
    y = torch.empty(total, dtype=torch.float32, device=dev)
    vt.vt_round_replay(torch.from_numpy(out[1][1]).to(dev), torch.from_numpy(idx.view(np.int32)).to(dev),
                       torch.from_numpy(dirw.view(np.int32)).to(dev), cnt, y)
    torch.cuda.synchronize()
    s = st.cpu().numpy().view(np.uint64)
    so = vo.threshold_stats(c64_T, out[1][1])
    assert int(s[0]) == so["n_flip"] and int(s[1]) == so["thr_flip"] and int(s[2]) == so["max_ulp64_diff"]
    assert np.array_equal(s[3:], so["hist"])
    assert max(so["thr_flip"], so["max_ulp64_diff"] + 1) <= 1 << 27      # tau = 1/4 ulp is safe for this pair
    assert np.array_equal(_bits(y.cpu().numpy()), _bits(c32_T))          # GPU auditor: 0 mismatches
    assert np.array_equal(_bits(vo.round_replay(out[1][1], idx, dirw)), _bits(c32_T))   # CPU replay of the same
    aud_rows = vo.gemm_f64(X[:16], W, bias=bias, order=1).ravel()        # CPU auditor on the first 16 rows
    k = int(np.searchsorted(idx, 16 * N))
    assert np.array_equal(_bits(vo.round_replay(aud_rows, idx[:k], dirw[:(k + 31) // 32], count=k)), _bits(c32_T[:16 * N]))


@pytest.mark.parametrize("thr,tau", [(32, 2.0 ** -24), (1, 2.0 ** -40), (1, 2.0 ** -32)])
def test_config5_full_size(thr, tau):
    """thr = 32 is tau = 2^-24 ulp; tau = 2^-40 and 2^-32 are below FP64 resolution and both quantise to thr = 1:
    exactly the planted ties are logged, the near misses one and two steps away are not."""
    import torch
    import paper_2403_09603_amd as vt
    dev = "cuda"
    n = 1 << 28
    assert vt.vt_thr_from_tau(tau) == thr
    x, kind = si.planted_vector(n, si.seed_for(5, 0), thr=thr)
    xa = si.perturb_steps(x, si.seed_for(5, 1), thr)
    xd = torch.from_numpy(x).to(dev)
    y = torch.empty(n, dtype=torch.float32, device=dev)
    log = vt.alloc_log(n // 4)
    ws = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_ROUND_LOG, 1, n))
    vt.vt_round_log(xd, tau, y, log, ws)
    torch.cuda.synchronize()
    cnt = int(log.count.item())
    assert 0 < cnt <= n // 4
    idx = log.idx.cpu().numpy().view(np.uint32)[:cnt]
    dirw = log.dir.cpu().numpy().view(np.uint32)[:(cnt + 31) // 32]
    yh = y.cpu().numpy()
    # properties at full size
    assert np.all(idx[1:] > idx[:-1]) and int(idx[-1]) < n
    logged = np.zeros(n, bool)
    logged[idx] = True
    assert logged[kind == 1].all() and not logged[kind == 2].any()
    assert np.array_equal(_dir_bits(dirw, cnt), (yh[idx].astype(np.float64) > x[idx]).astype(np.uint8))
    with np.errstate(over="ignore"):
        assert np.array_equal(_bits(yh), _bits(x.astype(np.float32)))      # library cast = round to nearest even
    # the oracle itself on sampled windows (tile and scan-round borders included)
    for lo in (0, 8192 * 1023 - 5000, n // 2 - 77777, n - (1 << 20)):
        hi = lo + (1 << 20)
        yo, io, do, co = vo.round_log(x[lo:hi], tau)
        a, b = np.searchsorted(idx, lo), np.searchsorted(idx, hi)
        assert b - a == co and np.array_equal(idx[a:b] - lo, io)
        assert np.array_equal(_dir_bits(dirw, cnt)[a:b], _dir_bits(do, co))
        assert np.array_equal(_bits(yh[lo:hi]), _bits(yo))
    # replay on the auditor's perturbed copy: identical to the trainer everywhere
    y2 = torch.empty(n, dtype=torch.float32, device=dev)
    xad = torch.from_numpy(xa).to(dev)
    vt.vt_round_replay(xad, log.idx, log.dir, cnt, y2)
    torch.cuda.synchronize()
    assert int((y2.view(torch.int32) != y.view(torch.int32)).sum().item()) == 0
    y2h = y2.cpu().numpy()
    lo, hi = n // 3, n // 3 + (1 << 20)
    a, b = int(np.searchsorted(idx, lo)), int(np.searchsorted(idx, hi))
    sub_dir = np.packbits(_dir_bits(dirw, cnt)[a:b], bitorder="little")
    sub_dir = np.frombuffer(sub_dir.tobytes().ljust(4 * ((b - a + 31) // 32), b"\0"), np.uint32)
    assert np.array_equal(_bits(y2h[lo:hi]), _bits(vo.round_replay(xa[lo:hi], idx[a:b] - lo, sub_dir, count=b - a)))
    st = torch.zeros(68, dtype=torch.int64, device=dev)
    vt.vt_threshold_stats(xd, xad, st)
    torch.cuda.synchronize()
    s = st.cpu().numpy().view(np.uint64)
    if thr == 1:
        # only exact ties are logged: the count is the number of planted values, every one a tie broken to even
        assert cnt == int((kind == 1).sum())
        assert np.array_equal(xa.view(np.uint64), x.view(np.uint64))       # no room to move inside (-1, 1) steps
        assert int(s[0]) == 0 and int(s[1]) == 0 and int(s[2]) == 0 and int(s[3]) == n
        return
    # without the log the auditor does diverge
    empty = vt.alloc_log(0)
    vt.vt_round_replay(xad, empty.idx, empty.dir, 0, y2)
    torch.cuda.synchronize()
    assert int((y2.view(torch.int32) != y.view(torch.int32)).sum().item()) > 1000
    # statistics of the pair at full size: every flip is inside the band, so thr_flip <= thr
    assert int(s[0]) > 1000 and 0 < int(s[1]) <= thr and int(s[2]) < thr and int(s[3:].sum()) == n

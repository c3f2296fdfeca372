"""GPU parity at the largest size the interface takes: n = 2^32 - 3 elements (log indices are 32-bit).

34 GB of FP64 input are drawn on the GPU (N(0,1), seeded) with exact FP32 midpoints planted at the
first and last element and on both sides of index 2^31.  The oracle checks three windows element by
element (start, around 2^31, ragged end): FP32 bits, the index entries that fall into the window,
their direction bits, and the bytes of the packed log.  Over the whole array: the number of logged
outputs against the definition evaluated with plain integer tensor operations (D = |r - 2^28| < thr on
the 29 dropped bits; every value is in the FP32-normal range), indices strictly ascending and below n,
replay of both log formats on the same data reproducing every FP32 bit, and the statistics of the
array against itself.
"""
import numpy as np
import pytest

from oracle import vt_oracle as vo

pytestmark = pytest.mark.gpu


@pytest.mark.timeout(900)
def test_round_log_replay_stats_at_the_index_limit():
    import torch
    import paper_2403_09603_amd as vt
    dev = "cuda"
    n = (1 << 32) - 3
    chunk = 1 << 28
    tau = 2.0 ** -7
    thr = vt.vt_thr_from_tau(tau)
    assert thr == 1 << 22
    gen = torch.Generator(device=dev)
    gen.manual_seed(0x240309603000 + 16 * 10)
    x = torch.empty(n, dtype=torch.float64, device=dev)
    for a in range(0, n, chunk):
        b = min(a + chunk, n)
        x[a:b] = torch.randn(b - a, generator=gen, device=dev, dtype=torch.float64)
    tie = 1.0 + 2.0 ** -24                                            # midway between two FP32 values
    planted = [0, (1 << 31) - 1, 1 << 31, n - 1]
    for i, p in enumerate(planted):
        x[p] = tie * (-1.0) ** i
    print("inputs drawn", flush=True)

    y = torch.empty(n, dtype=torch.float32, device=dev)
    cap = 80_000_000
    log = vt.alloc_log(cap)
    ws = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_ROUND_LOG, 1, n))
    vt.vt_round_log(x, tau, y, log, ws)
    torch.cuda.synchronize()
    count = int(log.count.item())
    print("round/log done, entries:", count, flush=True)

    # ---- whole array: count by the definition, order and range of the indices
    want = 0
    for a in range(0, n, chunk):
        r = x[a:min(a + chunk, n)].view(torch.int64) & ((1 << 29) - 1)
        want += int(((r - (1 << 28)).abs() < thr).sum().item())
    assert count == want and count <= cap and abs(count / n - 2 * tau) < 1e-4
    idx = log.idx[:count].to(torch.int64) & 0xFFFFFFFF
    assert bool((idx[1:] > idx[:-1]).all().item()) and int(idx[-1].item()) == n - 1 and int(idx[0].item()) == 0
    for p in planted:
        assert int(idx[torch.searchsorted(idx, torch.tensor([p], device=dev))].item()) == p      # ties are logged

    # ---- windows against the oracle
    win = 1 << 20
    starts = [0, (1 << 31) - win // 2, (n - win + 4) // 5 * 5]                  # multiples of 5; the last runs to the ragged end
    for a in starts:
        b = min(a + win, n)
        xw = x[a:b].cpu().numpy()
        yo, io, do, co = vo.round_log(xw, tau)
        assert np.array_equal(y[a:b].cpu().numpy().view(np.uint32), yo.view(np.uint32)), a
        lo, hi = (int(v) for v in torch.searchsorted(idx, torch.tensor([a, b], device=dev)).tolist())
        assert hi - lo == co and np.array_equal((idx[lo:hi] - a).cpu().numpy(), io.astype(np.int64)), a
        words = log.dir[lo >> 5:(hi + 31) >> 5].cpu().numpy().view(np.uint8)
        got = np.unpackbits(words, bitorder="little")[lo & 31:(lo & 31) + co]
        assert np.array_equal(got, np.unpackbits(do.view(np.uint8), bitorder="little")[:co]), a
    print("windows checked", flush=True)

    # ---- replay of the sparse log on the same data: every FP32 bit again
    y2 = torch.full((n,), float("nan"), dtype=torch.float32, device=dev)
    vt.vt_round_replay(x, log.idx, log.dir, count, y2)
    torch.cuda.synchronize()
    for a in range(0, n, chunk):
        b = min(a + chunk, n)
        assert torch.equal(y[a:b].view(torch.int32), y2[a:b].view(torch.int32)), a
    del idx, log
    print("sparse replay checked", flush=True)

    # ---- the packed log: same outputs and count, bytes of the windows, replay
    dlog = vt.alloc_dense_log(n)
    y2.fill_(float("nan"))
    vt.vt_round_log(x, tau, y2, dlog, ws)
    torch.cuda.synchronize()
    assert int(dlog.count.item()) == count and dlog.dense.numel() == (n + 4) // 5
    for a in range(0, n, chunk):
        b = min(a + chunk, n)
        assert torch.equal(y[a:b].view(torch.int32), y2[a:b].view(torch.int32)), a
    for a in starts:
        b = min(a + win, n)
        _, to, _ = vo.round_log_dense(x[a:b].cpu().numpy(), tau)
        assert np.array_equal(dlog.dense[a // 5:a // 5 + to.size].cpu().numpy(), to), a
    y2.fill_(float("nan"))
    vt.vt_round_replay_dense(x, dlog.dense, y2)
    torch.cuda.synchronize()
    for a in range(0, n, chunk):
        b = min(a + chunk, n)
        assert torch.equal(y[a:b].view(torch.int32), y2[a:b].view(torch.int32)), a
    print("packed log checked", flush=True)

    # ---- statistics of the array against itself: n identical pairs, nothing else
    out = torch.full((68,), -1, dtype=torch.int64, device=dev)
    vt.vt_threshold_stats(x, x, out)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert o[0] == 0 and o[1] == 0 and o[2] == 0 and o[3] == n and not o[4:].any()


@pytest.mark.timeout(900)
def test_batched_gemm_at_the_output_limit():
    """4095 products of 1024 x 64 by 64 x 1024 (the attention-score shape, B transposed): 2^32 - 2^20
    outputs, so the log indices, the bit-planes and the compaction run up to the 32-bit limit."""
    import torch
    import paper_2403_09603_amd as vt
    dev = "cuda"
    M = N = 1024
    K, batch = 64, 4095
    total = M * N * batch
    assert total < (1 << 32) <= total + M * N
    tau = 2.0 ** -7
    thr = vt.vt_thr_from_tau(tau)
    gen = torch.Generator(device=dev)
    gen.manual_seed(0x240309603000 + 16 * 10 + 1)
    A = torch.randn(batch, M, K, generator=gen, device=dev, dtype=torch.float64)
    B = torch.randn(batch, N, K, generator=gen, device=dev, dtype=torch.float64)
    C32 = torch.empty(total, dtype=torch.float32, device=dev)
    C64 = torch.empty(total, dtype=torch.float64, device=dev)
    cap = 80_000_000
    log = vt.alloc_log(cap)
    ws = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, M, N, K, batch))
    vt.vt_gemm_f64_round_log(False, True, M, N, K, 0.125, A, K, M * K, B, K, N * K, None, batch, C32, N, M * N, C64, 0, tau, log, ws)
    torch.cuda.synchronize()
    count = int(log.count.item())
    print("gemm done, entries:", count, flush=True)

    # ---- FP64 values of sampled rows against the oracle's extended-precision loops
    for b, i in [(0, 0), (2047, 1023), (2048, 0), (batch - 1, 1023), (1234, 567)]:
        a_row = A[b, i:i + 1].cpu().numpy()
        Bb = B[b].cpu().numpy()
        truth = vo.gemm_f64(a_row, Bb, transB=True, alpha=0.125, order=2)[0]
        got = C64[(b * M + i) * N:(b * M + i + 1) * N].cpu().numpy()
        bound = 1e-12 * 0.125 * np.linalg.norm(a_row) * np.linalg.norm(Bb, axis=1) + 1e-300
        assert np.all(np.abs(got - truth) <= bound), (b, i)

    # ---- whole output: count by the definition on the kernel's FP64 values, order of the indices
    want = 0
    step = 1 << 28
    for a in range(0, total, step):
        r = C64[a:min(a + step, total)].view(torch.int64) & ((1 << 29) - 1)
        want += int(((r - (1 << 28)).abs() < thr).sum().item())
    assert count == want and count <= cap
    idx = log.idx[:count].to(torch.int64) & 0xFFFFFFFF
    assert bool((idx[1:] > idx[:-1]).all().item()) and int(idx[-1].item()) < total and int(idx[-1].item()) > total - 1000

    # ---- windows (first matrix, both sides of index 2^31, the end) against the oracle's hook
    win = 1 << 20
    for a in (0, (1 << 31) - win // 2, total - win):
        b = a + win
        yo, io, do, co = vo.round_log(C64[a:b].cpu().numpy(), tau)
        assert np.array_equal(C32[a:b].cpu().numpy().view(np.uint32), yo.view(np.uint32)), a
        lo, hi = (int(v) for v in torch.searchsorted(idx, torch.tensor([a, b], device=dev)).tolist())
        assert hi - lo == co and np.array_equal((idx[lo:hi] - a).cpu().numpy(), io.astype(np.int64)), a
        words = log.dir[lo >> 5:(hi + 31) >> 5].cpu().numpy().view(np.uint8)
        got = np.unpackbits(words, bitorder="little")[lo & 31:(lo & 31) + co]
        assert np.array_equal(got, np.unpackbits(do.view(np.uint8), bitorder="little")[:co]), a

    # ---- replay of the log on the kernel's own FP64 values reproduces every FP32 output
    del A, B, idx
    y2 = torch.full((total,), float("nan"), dtype=torch.float32, device=dev)
    vt.vt_round_replay(C64, log.idx, log.dir, count, y2)
    torch.cuda.synchronize()
    for a in range(0, total, step):
        b = min(a + step, total)
        assert torch.equal(C32[a:b].view(torch.int32), y2[a:b].view(torch.int32)), a

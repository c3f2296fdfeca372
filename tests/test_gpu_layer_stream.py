"""GPU parity on a GPT-2 117M layer stream at reduced sequence length (the full-layer configuration).

One transformer block, d = 768, 12 heads of 64, T tokens of one sequence.  Every GEMM of the block
-- QKV 768->2304, the per-head scores Q K^T / 8 read as strided slices of the QKV output, P V
written head by head into the (T, 768) attention output, the output projection and the two MLP
projections -- goes through vt_gemm_f64_round_log; the element-wise steps between them are glue
(PyTorch FP64 on the GPU, identical for both parties) whose outputs go through vt_round_log.

For each GEMM: the FP64 values are checked against the oracle's extended-precision GEMM of the same
operands, the FP32 outputs and the log against the oracle's round/log of those FP64 values
(bit-exact), the per-layer threshold is chosen from vt_threshold_stats of the two accumulation
orders (checked against the oracle's statistics), and the auditor (variant 1 + vt_round_replay of
the trainer's log) must end with the trainer's FP32 bits.
"""
import numpy as np
import pytest

import paper_2403_09603_amd as vtlib
import synth_inputs as si
from oracle import vt_oracle as vo

pytestmark = pytest.mark.gpu

D, H, DH = 768, 12, 64


def _bits(y):
    return np.ascontiguousarray(y, np.float32).view(np.uint32)


class Party:
    """Calls into the library for one GEMM of the stream with explicit pitches and strides."""

    def __init__(self):
        import torch
        import paper_2403_09603_amd as vt
        self.torch, self.vt = torch, vt

    def gemm(self, A, lda, sA, B, ldb, sB, bias, M, N, K, batch, ldc, sC, out_elems, *, transB=False, alpha=1.0,
             variant=0, tau=0.0):
        torch, vt = self.torch, self.vt
        C32 = torch.full((out_elems,), float("nan"), dtype=torch.float32, device="cuda")
        C64 = torch.empty(batch * M * N, dtype=torch.float64, device="cuda")
        log = vt.alloc_log(batch * M * N)
        ws = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, M, N, K, batch))
        vt.vt_gemm_f64_round_log(False, transB, M, N, K, alpha, A, lda, sA, B, ldb, sB, bias, batch, C32, ldc, sC, C64,
                                 variant, tau, log, ws)
        torch.cuda.synchronize()
        cnt = int(log.count.item())
        return C32, C64, log, cnt

    def stats(self, y1, y2):
        torch = self.torch
        out = torch.zeros(68, dtype=torch.int64, device="cuda")
        self.vt.vt_threshold_stats(y1, y2, out)
        torch.cuda.synchronize()
        o = out.cpu().numpy().view(np.uint64)
        return {"n_flip": int(o[0]), "thr_flip": int(o[1]), "max_ulp64_diff": int(o[2]), "hist": o[3:].copy()}

    def replay(self, x64, log, cnt):
        torch = self.torch
        y = torch.empty(x64.numel(), dtype=torch.float32, device="cuda")
        self.vt.vt_round_replay(x64, log.idx, log.dir, cnt, y)
        torch.cuda.synchronize()
        return y

    def round_log(self, x64, tau):
        torch, vt = self.torch, self.vt
        y = torch.empty(x64.numel(), dtype=torch.float32, device="cuda")
        log = vt.alloc_log(x64.numel())
        ws = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_ROUND_LOG, 1, x64.numel()))
        vt.vt_round_log(x64.reshape(-1), tau, y, log, ws)
        torch.cuda.synchronize()
        return y, log, int(log.count.item())


def _host_operands(A, lda, sA, rows, cols, batch):
    """numpy copies of the `batch` (rows x cols) matrices a strided device operand describes."""
    flat = A.cpu().numpy()
    out = []
    for b in range(batch):
        base = b * sA
        out.append(np.lib.stride_tricks.as_strided(flat[base:], (rows, cols), (lda * 8, 8)).copy())
    return out


def _audited_gemm(P, name, A, lda, sA, B, ldb, sB, bias, M, N, K, batch, ldc, sC, out_elems, *, transB=False,
                  alpha=1.0):
    """Runs one GEMM of the stream for both parties; returns the (identical) FP32 output tensor."""
    kw = dict(transB=transB, alpha=alpha)
    _, c64_t, _, _ = P.gemm(A, lda, sA, B, ldb, sB, bias, M, N, K, batch, ldc, sC, out_elems, variant=0, **kw)
    _, c64_a, _, _ = P.gemm(A, lda, sA, B, ldb, sB, bias, M, N, K, batch, ldc, sC, out_elems, variant=1, **kw)
    # FP64 values of both orders against the oracle's extended-precision result
    hA = _host_operands(A, lda, sA, M, K, batch)
    hB = _host_operands(B, ldb, sB, N if transB else K, K if transB else N, batch)
    hb = bias.cpu().numpy() if bias is not None else None
    t64, a64 = c64_t.cpu().numpy().reshape(batch, M, N), c64_a.cpu().numpy().reshape(batch, M, N)
    for b in range(batch):
        truth = vo.gemm_f64(hA[b], hB[b], transB=transB, alpha=alpha, bias=hb, order=2)
        opB = hB[b].T if transB else hB[b]
        bound = 1e-12 * (abs(alpha) * np.linalg.norm(hA[b], axis=1)[:, None] * np.linalg.norm(opB, axis=0)[None, :]
                         + (np.abs(hb)[None, :] if hb is not None else 0.0)) + 1e-300
        assert np.all(np.abs(t64[b] - truth) <= bound), name
        assert np.all(np.abs(a64[b] - truth) <= bound), name
    # per-layer threshold from the statistics of the pair (checked against the oracle's)
    st = P.stats(c64_t, c64_a)
    so = vo.threshold_stats(t64.ravel(), a64.ravel())
    assert st["n_flip"] == so["n_flip"] and st["thr_flip"] == so["thr_flip"], name
    assert st["max_ulp64_diff"] == so["max_ulp64_diff"] and np.array_equal(st["hist"], so["hist"]), name
    thr = vtlib.vt_thr_layer_from_stats(st["thr_flip"], st["max_ulp64_diff"])      # the library's rule
    assert max(st["thr_flip"], st["max_ulp64_diff"] + 1) <= thr, name                # not capped at 1/4 ulp
    tau = thr * 2.0 ** -29
    c32_t, c64_t2, log, cnt = P.gemm(A, lda, sA, B, ldb, sB, bias, M, N, K, batch, ldc, sC, out_elems, variant=0,
                                     tau=tau, **kw)
    assert P.torch.equal(c64_t2, c64_t), name                     # same variant: same bits
    # trainer's FP32 outputs and log against the oracle's round/log of the same FP64 values
    yo, io, do, co = vo.round_log(t64.ravel(), tau)
    got = c32_t.cpu().numpy()
    dense = np.concatenate([np.lib.stride_tricks.as_strided(got[b * sC:], (M, N), (ldc * 4, 4)).ravel()
                            for b in range(batch)])
    assert np.array_equal(_bits(dense), _bits(yo)), name
    assert cnt == co and np.array_equal(log.idx.cpu().numpy().view(np.uint32)[:cnt], io), name
    nw = (cnt + 31) // 32
    if cnt:
        gd = np.unpackbits(log.dir.cpu().numpy().view(np.uint8)[:4 * nw], bitorder="little")[:cnt]
        od = np.unpackbits(do.view(np.uint8)[:4 * nw], bitorder="little")[:cnt]
        assert np.array_equal(gd, od), name
    # auditor: its own FP64 values + the trainer's log
    y_a = P.replay(c64_a, log, cnt).cpu().numpy()
    assert np.array_equal(_bits(y_a), _bits(yo)), name
    return c32_t, {"name": name, "thr": thr, "logged": cnt, "n_flip": st["n_flip"]}


def _audited_elementwise(P, name, x64, tau=2.0 ** -29):
    """Glue output -> FP32 through the standalone hook; both parties hold the same FP64 values here,
    so the log only has to reproduce plain rounding; checked against the oracle all the same."""
    y, log, cnt = P.round_log(x64, tau)
    yo, io, do, co = vo.round_log(x64.cpu().numpy().ravel(), tau)
    assert cnt == co and np.array_equal(_bits(y.cpu().numpy()), _bits(yo)), name
    assert np.array_equal(log.idx.cpu().numpy().view(np.uint32)[:cnt], io), name
    y_a = P.replay(x64.reshape(-1), log, cnt)
    assert np.array_equal(_bits(y_a.cpu().numpy()), _bits(yo)), name
    return y


def _audited_layer(P, name, op, a, b, gamma, beta, rows, cols, **kw):
    """One fused element-wise / row-wise layer for both parties (two summation orders of the row
    statistics); FP64 values against the oracle, hook outputs bit-exact, per-layer threshold, replay."""
    torch, vt = P.torch, P.vt
    n = rows * cols

    def run(variant, tau):
        y = torch.empty(n, dtype=torch.float32, device="cuda")
        y64 = torch.empty(n, dtype=torch.float64, device="cuda")
        log = vt.alloc_log(n)
        ws = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_LAYER_ROUND_LOG, rows, cols))
        vt.vt_layer_f64_round_log(op, a, b, gamma, beta, rows, cols, y, y64, variant, tau, log, ws, **kw)
        torch.cuda.synchronize()
        return y, y64, log, int(log.count.item())

    _, t64, _, _ = run(0, 0.0)
    _, a64, _, _ = run(1, 0.0)
    ha = a.cpu().numpy().reshape(rows, cols)
    if op == vt.VT_LAYER_NORM:
        truth = vo.layernorm(ha, gamma.cpu().numpy() if gamma is not None else None,
                             beta.cpu().numpy() if beta is not None else None, kw.get("eps", 1e-5), order=2)
    elif op == vt.VT_LAYER_SOFTMAX:
        truth = vo.softmax(ha, kw.get("scale", 1.0), kw.get("causal_period", 0), order=2)
    elif op == vt.VT_LAYER_ADD:
        truth = vo.elementwise(vo.EW_ADD, ha, b.cpu().numpy().reshape(rows, cols), exact=True)
    else:
        truth = vo.elementwise(vo.EW_GELU_TANH, ha, exact=True)
    tol = 2.0 ** -52 * (8 + 4 * np.sqrt(cols)) * (np.abs(truth) + (1.0 if op == vt.VT_LAYER_NORM else 0.0) + np.abs(ha) * (op == vt.VT_LAYER_GELU_TANH)) + 1e-300
    for v64 in (t64, a64):
        assert np.all(np.abs(v64.cpu().numpy().reshape(rows, cols) - truth) <= tol), name
    st = P.stats(t64, a64)
    thr = vtlib.vt_thr_layer_from_stats(st["thr_flip"], st["max_ulp64_diff"])      # the library's rule
    assert max(st["thr_flip"], st["max_ulp64_diff"] + 1) <= thr, name                # not capped at 1/4 ulp
    tau = thr * 2.0 ** -29
    y, t64b, log, cnt = run(0, tau)
    assert torch.equal(t64b, t64), name
    yo, io, do, co = vo.round_log(t64.cpu().numpy(), tau)
    assert cnt == co and np.array_equal(_bits(y.cpu().numpy()), _bits(yo)), name
    assert np.array_equal(log.idx.cpu().numpy().view(np.uint32)[:cnt], io), name
    assert np.array_equal(_bits(P.replay(a64, log, cnt).cpu().numpy()), _bits(yo)), name     # auditor == trainer
    return y


def test_gpt2_block_stream_through_the_library_alone():
    """The same block with its layer norms, softmax, GELU and residual additions as fused layer +
    hook calls: no FP64 intermediate of the block is produced outside the library."""
    import torch
    P = Party()
    vt = P.vt
    T = 136
    g = si.rng(si.seed_for(3, 2))

    def param(shape, sigma=0.02, shift=0.0):
        return torch.from_numpy((g.standard_normal(shape) * sigma + shift).astype(np.float32).astype(np.float64)).cuda()

    def f64(t32):
        return t32.to(torch.float64)

    x = param((T, D), 1.0).reshape(-1)
    g1, be1, g2, be2 = param(D, 0.1, 1.0), param(D, 0.1), param(D, 0.1, 1.0), param(D, 0.1)
    Wqkv, bqkv, Wo, bo = param((D, 3 * D)), param(3 * D), param((D, D)), param(D)
    W1, b1, W2, b2 = param((D, 4 * D)), param(4 * D), param((4 * D, D)), param(D)
    h = _audited_layer(P, "ln1", vt.VT_LAYER_NORM, x, None, g1, be1, T, D, eps=1e-5)
    qkv32, _ = _audited_gemm(P, "qkv", f64(h), D, 0, Wqkv.reshape(-1), 3 * D, 0, bqkv, T, 3 * D, D, 1, 3 * D, 0, T * 3 * D)
    qkv = f64(qkv32)
    s32, _ = _audited_gemm(P, "scores", qkv, 3 * D, DH, qkv[D:], 3 * D, DH, None, T, T, DH, H, T, T * T, H * T * T,
                           transB=True, alpha=0.125)
    # rows are (head, token): row r attends to columns <= r mod T
    p32 = _audited_layer(P, "softmax", vt.VT_LAYER_SOFTMAX, f64(s32), None, None, None, H * T, T, scale=1.0, causal_period=T)
    o32, _ = _audited_gemm(P, "pv", f64(p32), T, T * T, qkv[2 * D:], 3 * D, DH, None, T, DH, T, H, D, DH, T * D)
    a32, _ = _audited_gemm(P, "attn_out", f64(o32), D, 0, Wo.reshape(-1), D, 0, bo, T, D, D, 1, D, 0, T * D)
    x1 = _audited_layer(P, "residual1", vt.VT_LAYER_ADD, x, f64(a32), None, None, T, D)
    h2 = _audited_layer(P, "ln2", vt.VT_LAYER_NORM, f64(x1), None, g2, be2, T, D, eps=1e-5)
    u32_, _ = _audited_gemm(P, "mlp_up", f64(h2), D, 0, W1.reshape(-1), 4 * D, 0, b1, T, 4 * D, D, 1, 4 * D, 0, T * 4 * D)
    act = _audited_layer(P, "gelu", vt.VT_LAYER_GELU_TANH, f64(u32_), None, None, None, T, 4 * D)
    d32, _ = _audited_gemm(P, "mlp_down", f64(act), 4 * D, 0, W2.reshape(-1), D, 0, b2, T, D, 4 * D, 1, D, 0, T * D)
    out = _audited_layer(P, "residual2", vt.VT_LAYER_ADD, f64(x1), f64(d32), None, None, T, D)
    assert torch.isfinite(out).all()
    # the causal mask reached the probabilities: strictly upper triangle is exactly zero
    pm = p32.reshape(H, T, T)
    assert (pm.triu(1) == 0).all() and (pm.diagonal(dim1=1, dim2=2) > 0).all()


@pytest.mark.parametrize("T", [200])
def test_gpt2_block_stream(T):
    import torch
    P = Party()
    g = si.rng(si.seed_for(3, 1))
    dev = "cuda"

    def param(shape, sigma=0.02):
        return torch.from_numpy((g.standard_normal(shape) * sigma).astype(np.float32).astype(np.float64)).to(dev)

    x = torch.from_numpy(g.standard_normal((T, D)).astype(np.float32).astype(np.float64)).to(dev)
    Wqkv, bqkv = param((D, 3 * D)), param((3 * D,))
    Wo, bo = param((D, D)), param((D,))
    W1, b1 = param((D, 4 * D)), param((4 * D,))
    W2, b2 = param((4 * D, D)), param((D,))
    report = []

    def f64(t32):
        return t32.to(torch.float64)

    h = _audited_elementwise(P, "ln1", torch.nn.functional.layer_norm(x, (D,)))
    h64 = f64(h).reshape(-1)
    qkv32, r = _audited_gemm(P, "qkv", h64, D, 0, Wqkv.reshape(-1), 3 * D, 0, bqkv, T, 3 * D, D, 1, 3 * D, 0, T * 3 * D)
    report.append(r)
    qkv = f64(qkv32)                                        # (T * 2304,) flat, row pitch 2304
    # scores per head: A = Q slice (pitch 2304, heads 64 apart), B = K slice stored (T x 64) -> transB
    s32, r = _audited_gemm(P, "scores", qkv, 3 * D, DH, qkv[D:], 3 * D, DH, None, T, T, DH, H, T, T * T, H * T * T,
                           transB=True, alpha=0.125)
    report.append(r)
    s = f64(s32).reshape(H, T, T)
    mask = torch.ones(T, T, dtype=torch.bool, device=dev).tril()
    p = torch.softmax(s.masked_fill(~mask, float("-inf")), dim=-1)
    p32 = _audited_elementwise(P, "softmax", p)
    p64 = f64(p32)
    # P V per head, written straight into the (T, 768) attention output: ldc = 768, heads 64 apart
    o32, r = _audited_gemm(P, "pv", p64, T, T * T, qkv[2 * D:], 3 * D, DH, None, T, DH, T, H, D, DH, T * D)
    report.append(r)
    assert not torch.isnan(o32).any()                       # every column of the shared output was written
    a32, r = _audited_gemm(P, "attn_out", f64(o32), D, 0, Wo.reshape(-1), D, 0, bo, T, D, D, 1, D, 0, T * D)
    report.append(r)
    x1 = _audited_elementwise(P, "residual1", x + f64(a32).reshape(T, D))
    h2 = _audited_elementwise(P, "ln2", torch.nn.functional.layer_norm(f64(x1).reshape(T, D), (D,)))
    u32_, r = _audited_gemm(P, "mlp_up", f64(h2), D, 0, W1.reshape(-1), 4 * D, 0, b1, T, 4 * D, D, 1, 4 * D, 0, T * 4 * D)
    report.append(r)
    act = _audited_elementwise(P, "gelu", torch.nn.functional.gelu(f64(u32_)))
    d32, r = _audited_gemm(P, "mlp_down", f64(act), 4 * D, 0, W2.reshape(-1), D, 0, b2, T, D, 4 * D, 1, D, 0, T * D)
    report.append(r)
    _audited_elementwise(P, "residual2", f64(x1).reshape(T, D) + f64(d32).reshape(T, D))
    assert [r["name"] for r in report] == ["qkv", "scores", "pv", "attn_out", "mlp_up", "mlp_down"]
    assert all(r["logged"] > 0 for r in report)

"""numpy-in / numpy-out wrappers around the HIP library for the GPU parity tests.
Everything computed here goes through the C ABI (paper_2403_09603_amd.binding)."""
import numpy as np
import torch

import paper_2403_09603_amd as vt

DEV = "cuda"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def u32(t):
    return t.cpu().numpy().view(np.uint32)


def gpu_round_log(x, tau, cap=None, misalign=False, b_r=32):
    """misalign=True places x on an 8-byte (not 16-byte) boundary, which makes the library take
    its bit-plane + compaction path instead of the single-pass kernel."""
    x = np.ascontiguousarray(x, np.float64).ravel()
    n = x.size
    cap = n if cap is None else cap
    if misalign:
        buf = torch.empty(n + 1, dtype=torch.float64, device=DEV)
        xd = buf[1:]
        if n:
            xd.copy_(torch.from_numpy(x))
        assert n == 0 or xd.data_ptr() % 16 == 8
    else:
        xd = dev(x) if n else torch.empty(0, dtype=torch.float64, device=DEV)
    y = torch.empty(n, dtype=torch.float32, device=DEV)
    log = vt.alloc_log(cap)
    log.b_r = b_r
    ws = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_ROUND_LOG, 1, n))
    vt.vt_round_log(xd, tau, y, log, ws)
    torch.cuda.synchronize()
    count = int(log.count.item())
    k = min(count, cap)
    return (y.cpu().numpy(), u32(log.idx)[:k].copy(), u32(log.dir)[:(k + 31) // 32].copy(), count)


def gpu_round_replay(x, idx, dirw, count=None, misalign=False, b_r=32):
    x = np.ascontiguousarray(x, np.float64).ravel()
    count = len(idx) if count is None else count
    if misalign:
        buf = torch.empty(x.size + 1, dtype=torch.float64, device=DEV)
        xd = buf[1:]
        xd.copy_(torch.from_numpy(x))
    else:
        xd = dev(x)
    y = torch.empty(x.size, dtype=torch.float32, device=DEV)
    idx_d = dev(np.ascontiguousarray(idx, np.uint32).view(np.int32)) if len(idx) else torch.zeros(1, dtype=torch.int32, device=DEV)
    dir_d = dev(np.ascontiguousarray(dirw, np.uint32).view(np.int32)) if len(dirw) else torch.zeros(1, dtype=torch.int32, device=DEV)
    vt.vt_round_replay(xd, idx_d, dir_d, count, y, b_r=b_r)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def gpu_stats(y1, y2, b_r=32):
    out = torch.full((68,), -1, dtype=torch.int64, device=DEV)
    vt.vt_threshold_stats(dev(np.ascontiguousarray(y1, np.float64).ravel()),
                          dev(np.ascontiguousarray(y2, np.float64).ravel()), out, b_r=b_r)
    torch.cuda.synchronize()
    o = out.cpu().numpy().view(np.uint64)
    return {"n_flip": int(o[0]), "thr_flip": int(o[1]), "max_ulp64_diff": int(o[2]), "hist": o[3:].copy()}


def gpu_gemm(A, B, *, transA=False, transB=False, alpha=1.0, bias=None, tau=0.0, variant=0, cap=None,
             want_c64=True, ldc=None, b_r=32):
    """A, B: numpy arrays as stored, 2-D (or 3-D with a leading batch dimension)."""
    A = np.ascontiguousarray(A, np.float64)
    B = np.ascontiguousarray(B, np.float64)
    batch = A.shape[0] if A.ndim == 3 else 1
    a2, b2 = A.shape[-2:], B.shape[-2:]
    M, K = (a2[1], a2[0]) if transA else a2
    K2, N = (b2[1], b2[0]) if transB else b2
    assert K == K2
    strideA = a2[0] * a2[1] if A.ndim == 3 else 0
    strideB = b2[0] * b2[1] if B.ndim == 3 else 0
    ldc = N if ldc is None else ldc
    total = batch * M * N
    cap = total if cap is None else cap
    Ad, Bd = dev(A), dev(B)
    C32 = torch.full((batch, M, ldc), float("nan"), dtype=torch.float32, device=DEV)
    C64 = torch.empty((batch, M, N), dtype=torch.float64, device=DEV) if want_c64 else None
    log = vt.alloc_log(cap)
    log.b_r = b_r
    op = vt.VT_OP_GEMM_ROUND_LOG if b_r == 32 else vt.VT_OP_GEMM_ROUND_LOG_BR
    ws = vt.alloc_workspace(vt.vt_workspace_bytes(op, M, N, K, batch))
    bias_d = dev(np.ascontiguousarray(bias, np.float64)) if bias is not None else None
    vt.vt_gemm_f64_round_log(transA, transB, M, N, K, alpha, Ad, a2[1], strideA, Bd, b2[1], strideB, bias_d, batch,
                             C32, ldc, M * ldc, C64, variant, tau, log, ws)
    torch.cuda.synchronize()
    count = int(log.count.item())
    k = min(count, cap)
    return {"C32": C32.cpu().numpy()[:, :, :N].reshape(batch, M, N), "C32_full": C32.cpu().numpy(),
            "C64": C64.cpu().numpy() if want_c64 else None,
            "idx": u32(log.idx)[:k].copy(), "dir": u32(log.dir)[:(k + 31) // 32].copy(), "count": count}


def gpu_conv(mode, X, B, KH, KW, *, stride=1, pad=0, dil=1, bias=None, tau=0.0, variant=0, misalign=False, b_r=32,
             xshape=None, dense=False):
    """mode 0: forward, B = weights (KH,KW,C,Cout); mode 1: weight gradient, B = dY (N,Ho,Wo,Cout).
    X is (N,H,W,C).  mode 2: input gradient, X = dY (N,Ho,Wo,Cout), B = weights, xshape = (N,H,W,C).
    misalign=True puts X on an 8-byte (not 16-byte) boundary.  dense=True asks for the packed ternary log."""
    pair = lambda v: (int(v), int(v)) if np.isscalar(v) else (int(v[0]), int(v[1]))
    (sh, sw), (ph, pw), (dh, dw) = pair(stride), pair(pad), pair(dil)
    X = np.ascontiguousarray(X, np.float64)
    B = np.ascontiguousarray(B, np.float64)
    N, H, W, Cin = X.shape if mode != 2 else xshape
    Cout = B.shape[-1]
    d = vt.Conv2d(N, H, W, Cin, KH, KW, sh, sw, ph, pw, dh, dw)
    M, Nn, K = vt.vt_conv2d_gemm_shape(d, Cout, mode)
    if misalign:
        buf = torch.empty(X.size + 1, dtype=torch.float64, device=DEV)
        Xd = buf[1:]
        Xd.copy_(torch.from_numpy(X.ravel()))
        assert Xd.data_ptr() % 16 == 8
    else:
        Xd = dev(X.ravel())
    Bd = dev(B.ravel())
    C32 = torch.full((max(M * Nn, 1),), float("nan"), dtype=torch.float32, device=DEV)
    C64 = torch.empty(max(M * Nn, 1), dtype=torch.float64, device=DEV)
    log = vt.alloc_dense_log(M * Nn) if dense else vt.alloc_log(M * Nn)
    log.b_r = b_r
    if dense:
        log.dense.fill_(0xEE)
    if mode == 2:
        op = vt.VT_OP_CONV_DGRAD_ROUND_LOG if b_r == 32 else vt.VT_OP_CONV_DGRAD_ROUND_LOG_BR
    else:
        op = vt.VT_OP_GEMM_ROUND_LOG if b_r == 32 else vt.VT_OP_GEMM_ROUND_LOG_BR
    ws = vt.alloc_workspace(vt.vt_workspace_bytes(op, M, Nn, K, 1))
    bias_d = dev(np.ascontiguousarray(bias, np.float64)) if bias is not None else None
    vt.vt_conv2d_f64_round_log(mode, d, Cout, Xd, Bd, bias_d, C32, C64, variant, tau, log, ws)
    torch.cuda.synchronize()
    count = int(log.count.item())
    if dense:
        full = log.dense.cpu().numpy()
        assert (full[(M * Nn + 4) // 5:] == 0xEE).all()
        return {"C32": C32.cpu().numpy()[:M * Nn].reshape(M, Nn), "C64": C64.cpu().numpy()[:M * Nn].reshape(M, Nn),
                "tlog": full[:(M * Nn + 4) // 5].copy(), "count": count, "shape": (M, Nn, K)}
    return {"C32": C32.cpu().numpy()[:M * Nn].reshape(M, Nn), "C64": C64.cpu().numpy()[:M * Nn].reshape(M, Nn),
            "idx": u32(log.idx)[:count].copy(), "dir": u32(log.dir)[:(count + 31) // 32].copy(), "count": count,
            "shape": (M, Nn, K)}


def gpu_round_log_dense(x, tau, misalign=False, b_r=32):
    """Standalone trainer hook writing the packed ternary log: (y, tlog bytes, n_logged)."""
    x = np.ascontiguousarray(x, np.float64).ravel()
    n = x.size
    if misalign:
        buf = torch.empty(n + 1, dtype=torch.float64, device=DEV)
        xd = buf[1:]
        if n:
            xd.copy_(torch.from_numpy(x))
    else:
        xd = dev(x) if n else torch.empty(0, dtype=torch.float64, device=DEV)
    y = torch.empty(n, dtype=torch.float32, device=DEV)
    log = vt.alloc_dense_log(n)
    log.b_r = b_r
    log.dense.fill_(0xEE)
    log.count.fill_(-1)
    ws = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_ROUND_LOG, 1, n))
    vt.vt_round_log(xd, tau, y, log, ws)
    torch.cuda.synchronize()
    full = log.dense.cpu().numpy()
    assert (full[(n + 4) // 5:] == 0xEE).all()               # nothing written past the log
    return y.cpu().numpy(), full[:(n + 4) // 5].copy(), int(log.count.item())


def gpu_round_replay_dense(x, tlog, misalign=False, b_r=32):
    x = np.ascontiguousarray(x, np.float64).ravel()
    if misalign:
        buf = torch.empty(x.size + 1, dtype=torch.float64, device=DEV)
        xd = buf[1:]
        xd.copy_(torch.from_numpy(x))
    else:
        xd = dev(x) if x.size else torch.empty(0, dtype=torch.float64, device=DEV)
    t = np.ascontiguousarray(tlog, np.uint8)
    td = dev(t) if t.size else torch.zeros(4, dtype=torch.uint8, device=DEV)
    y = torch.empty(x.size, dtype=torch.float32, device=DEV)
    vt.vt_round_replay_dense(xd, td, y, b_r=b_r)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def gpu_gemm_dense(A, B, *, transA=False, transB=False, alpha=1.0, bias=None, tau=0.0, variant=0, ldc=None, b_r=32):
    """GEMM entry point with the packed ternary log as output format."""
    A = np.ascontiguousarray(A, np.float64)
    B = np.ascontiguousarray(B, np.float64)
    batch = A.shape[0] if A.ndim == 3 else 1
    a2, b2 = A.shape[-2:], B.shape[-2:]
    M, K = (a2[1], a2[0]) if transA else a2
    K2, N = (b2[1], b2[0]) if transB else b2
    assert K == K2
    strideA = a2[0] * a2[1] if A.ndim == 3 else 0
    strideB = b2[0] * b2[1] if B.ndim == 3 else 0
    ldc = N if ldc is None else ldc
    total = batch * M * N
    C32 = torch.full((batch, M, ldc), float("nan"), dtype=torch.float32, device=DEV)
    C64 = torch.empty((batch, M, N), dtype=torch.float64, device=DEV)
    log = vt.alloc_dense_log(total)
    log.b_r = b_r
    log.dense.fill_(0xEE)
    ws = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG if b_r == 32 else vt.VT_OP_GEMM_ROUND_LOG_BR,
                                                  M, N, K, batch))
    bias_d = dev(np.ascontiguousarray(bias, np.float64)) if bias is not None else None
    vt.vt_gemm_f64_round_log(transA, transB, M, N, K, alpha, dev(A), a2[1], strideA, dev(B), b2[1], strideB, bias_d, batch,
                             C32, ldc, M * ldc, C64, variant, tau, log, ws)
    torch.cuda.synchronize()
    full = log.dense.cpu().numpy()
    assert (full[max((total + 4) // 5, 0):] == 0xEE).all()
    return {"C32": C32.cpu().numpy()[:, :, :N].reshape(batch, M, N), "C64": C64.cpu().numpy(),
            "tlog": full[:(total + 4) // 5].copy(), "count": int(log.count.item())}


def gpu_layer(op, a, b=None, gamma=None, beta=None, *, eps=1e-5, scale=1.0, causal_period=0, tau=0.0, variant=0,
              dense=False, b_r=32, want_y64=True, cap=None):
    """Fused layer + trainer hook.  a (and b): 2-D numpy arrays.  Returns y32, y64 (unless want_y64 is
    False: the call then gets no FP64 debug buffer, as in the benchmarks) and the log (index list of
    capacity `cap`, default one entry per output)."""
    a = np.ascontiguousarray(a, np.float64)
    rows, cols = a.shape
    n = rows * cols
    ad = dev(a.ravel()) if n else torch.empty(0, dtype=torch.float64, device=DEV)
    bd = dev(np.ascontiguousarray(b, np.float64).ravel()) if b is not None else None
    gd = dev(np.ascontiguousarray(gamma, np.float64)) if gamma is not None else None
    be = dev(np.ascontiguousarray(beta, np.float64)) if beta is not None else None
    y = torch.full((max(n, 1),), float("nan"), dtype=torch.float32, device=DEV)
    y64 = torch.full((max(n, 1),), float("nan"), dtype=torch.float64, device=DEV)
    log = vt.alloc_dense_log(n) if dense else vt.alloc_log(n if cap is None else cap)
    log.b_r = b_r
    ws = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_LAYER_ROUND_LOG, rows, cols))
    vt.vt_layer_f64_round_log(op, ad, bd, gd, be, rows, cols, y, y64 if want_y64 else None, variant, tau, log, ws, eps=eps,
                              scale=scale, causal_period=causal_period)
    torch.cuda.synchronize()
    cnt = int(log.count.item())
    out = {"y32": y.cpu().numpy()[:n].reshape(rows, cols), "count": cnt}
    if want_y64:
        out["y64"] = y64.cpu().numpy()[:n].reshape(rows, cols)
    if dense:
        out["tlog"] = log.dense.cpu().numpy()[:(n + 4) // 5].copy()
    else:
        stored = cnt if cap is None else min(cnt, cap)
        out["idx"] = u32(log.idx)[:stored].copy()
        out["dir"] = u32(log.dir)[:(stored + 31) // 32].copy()
    return out

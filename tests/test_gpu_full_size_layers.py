"""GPU parity at full size for the layer shapes of the GPT-2 117M stream (batch 8 x 1024 tokens) and of
ResNet-50 at batch 64: FP64 values against the oracle on sampled outputs (the oracle computes them one
by one), and everything after the FP64 value -- all FP32 outputs, the whole log -- bit-exact against
the oracle's round/log of the kernel's own FP64 values.  Inputs are seeded and synthetic with the
shapes and value distributions of those layers (N(0,1) activations rounded to FP32, N(0, 0.02^2)
weights; U(0,1) images, post-ReLU activations, He-normal filters)."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import vt_oracle as vo

pytestmark = pytest.mark.gpu


def _bits(y):
    return np.ascontiguousarray(y, np.float32).view(np.uint32)


def _dir_bits(dirw, count):
    return np.unpackbits(np.ascontiguousarray(dirw, np.uint32).view(np.uint8), bitorder="little")[:count]


def _f32grid(a):
    return a.astype(np.float32).astype(np.float64)


def _hook_parity(c32, c64, log, cnt, tau):
    yo, io, do, co = vo.round_log(c64.ravel(), tau)
    assert cnt == co
    assert np.array_equal(_bits(c32.ravel()), _bits(yo))
    assert np.array_equal(log.idx.cpu().numpy().view(np.uint32)[:cnt], io)
    assert np.array_equal(_dir_bits(log.dir.cpu().numpy().view(np.uint32)[:(cnt + 31) // 32], cnt), _dir_bits(do, co))


@pytest.mark.parametrize("name,M,N,K", [("qkv", 8192, 2304, 768), ("attn_out", 8192, 768, 768),
                                        ("mlp_down", 8192, 768, 3072)])
def test_gpt2_linear_layers_full_size(name, M, N, K):
    import torch
    import paper_2403_09603_amd as vt
    g = si.rng(si.seed_for(3, 20) + N + K)
    X = _f32grid(g.standard_normal((M, K)))
    W = _f32grid(g.standard_normal((K, N)) * 0.02)
    bias = _f32grid(g.standard_normal(N) * 0.02)
    tau = 2.0 ** -5
    Xd, Wd, bd = (torch.from_numpy(a).cuda() for a in (X, W, bias))
    C32 = torch.empty(M * N, dtype=torch.float32, device="cuda")
    C64 = torch.empty(M * N, dtype=torch.float64, device="cuda")
    log = vt.alloc_log(M * N)
    ws = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, M, N, K, 1))
    vt.vt_gemm_f64_round_log(False, False, M, N, K, 1.0, Xd, K, 0, Wd, N, 0, bd, 1, C32, N, 0, C64, 0, tau, log, ws)
    torch.cuda.synchronize()
    c64 = C64.cpu().numpy().reshape(M, N)
    wn = np.linalg.norm(W, axis=0)
    for r in [0, 63, 64, 127, 128, 8191] + list(g.integers(0, M, 8)):
        truth = vo.gemm_f64(X[r:r + 1], W, bias=bias, order=2)[0]
        assert np.all(np.abs(c64[r] - truth) <= 1e-12 * (np.linalg.norm(X[r]) * wn + np.abs(bias)) + 1e-300), name
    _hook_parity(C32.cpu().numpy(), c64, log, int(log.count.item()), tau)


def test_gpt2_attention_scores_and_pv_full_size():
    """One sequence of 1024 tokens, 12 heads: scores and P V read their operands as strided slices of
    the (1024, 2304) QKV output; P V writes head by head into the (1024, 768) attention output."""
    import torch
    import paper_2403_09603_amd as vt
    T, D, H, DH = 1024, 768, 12, 64
    g = si.rng(si.seed_for(3, 30))
    qkv = _f32grid(g.standard_normal((T, 3 * D)))
    qkv_d = torch.from_numpy(qkv).cuda().reshape(-1)
    tau = 2.0 ** -5
    # scores: batch = heads, A = Q slice, B = K slice (stored T x 64: transB), alpha = 1/8
    S32 = torch.empty(H * T * T, dtype=torch.float32, device="cuda")
    S64 = torch.empty(H * T * T, dtype=torch.float64, device="cuda")
    log = vt.alloc_log(H * T * T)
    ws = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, T, T, DH, H))
    vt.vt_gemm_f64_round_log(False, True, T, T, DH, 0.125, qkv_d, 3 * D, DH, qkv_d[D:], 3 * D, DH, None, H, S32, T, T * T,
                             S64, 0, tau, log, ws)
    torch.cuda.synchronize()
    s64 = S64.cpu().numpy().reshape(H, T, T)
    for h, r in [(0, 0), (0, 1023), (5, 64), (11, 127), (11, 1023)] + [tuple(v) for v in g.integers(0, [H, T], (6, 2))]:
        q = qkv[r:r + 1, h * DH:(h + 1) * DH]
        kmat = np.ascontiguousarray(qkv[:, D + h * DH: D + (h + 1) * DH])
        truth = vo.gemm_f64(q, kmat, transB=True, alpha=0.125, order=2)[0]
        assert np.all(np.abs(s64[h, r] - truth) <= 1e-12 * 0.125 * np.linalg.norm(q) * np.linalg.norm(kmat, axis=1) + 1e-300)
    _hook_parity(S32.cpu().numpy(), s64, log, int(log.count.item()), tau)
    # P V: P = row-softmax of the rounded scores (glue), FP32 grid; output pitch 768, heads 64 apart
    P = torch.softmax(S32.reshape(H, T, T).to(torch.float64), dim=-1).to(torch.float32).to(torch.float64).reshape(-1)
    O32 = torch.full((T * D,), float("nan"), dtype=torch.float32, device="cuda")
    O64 = torch.empty(H * T * DH, dtype=torch.float64, device="cuda")
    log2 = vt.alloc_log(H * T * DH)
    ws2 = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, T, DH, T, H))
    vt.vt_gemm_f64_round_log(False, False, T, DH, T, 1.0, P, T, T * T, qkv_d[2 * D:], 3 * D, DH, None, H, O32, D, DH, O64,
                             0, tau, log2, ws2)
    torch.cuda.synchronize()
    o64 = O64.cpu().numpy().reshape(H, T, DH)
    Ph = P.cpu().numpy().reshape(H, T, T)
    for h, r in [(0, 0), (3, 500), (11, 1023)]:
        vmat = np.ascontiguousarray(qkv[:, 2 * D + h * DH: 2 * D + (h + 1) * DH])
        truth = vo.gemm_f64(Ph[h, r:r + 1], vmat, order=2)[0]
        assert np.all(np.abs(o64[h, r] - truth) <= 1e-12 * np.linalg.norm(Ph[h, r]) * np.linalg.norm(vmat, axis=0) + 1e-300)
    o32 = O32.cpu().numpy().reshape(T, H, DH).transpose(1, 0, 2)          # (head, token, 64): the log's order
    assert not np.isnan(o32).any()
    _hook_parity(np.ascontiguousarray(o32), o64, log2, int(log2.count.item()), tau)


@pytest.mark.parametrize("name,geom", [
    ("conv1 7x7/2, 3 channels", (64, 224, 224, 3, 7, 7, 64, 2, 3)),
    ("3x3 bottleneck", (64, 56, 56, 64, 3, 3, 64, 1, 1)),
    ("1x1/2 downsample", (64, 56, 56, 256, 1, 1, 512, 2, 0)),
])
def test_resnet_convolutions_full_size(name, geom):
    import torch
    import paper_2403_09603_amd as vt
    N, H, W, Cin, KH, KW, Cout, stride, pad = geom
    g = si.rng(si.seed_for(4, 40) + H + Cin)
    X = g.random((N, H, W, Cin)) if Cin == 3 else np.maximum(g.standard_normal((N, H, W, Cin)), 0.0)
    X = _f32grid(X)
    Wt = _f32grid(g.standard_normal((KH, KW, Cin, Cout)) * np.sqrt(2.0 / (KH * KW * Cin)))
    tau = 2.0 ** -5
    d = vt.Conv2d(N, H, W, Cin, KH, KW, stride, stride, pad, pad, 1, 1)
    _, Ho, Wo = vo.conv2d_geometry(X.shape, KH, KW, stride, pad, 1)
    Xd, Wd = torch.from_numpy(X).cuda().reshape(-1), torch.from_numpy(Wt).cuda().reshape(-1)
    # ---- forward
    M, Nn, K = vt.vt_conv2d_gemm_shape(d, Cout, vt.VT_CONV_FORWARD)
    assert (M, Nn, K) == (N * Ho * Wo, Cout, KH * KW * Cin)
    Y32 = torch.empty(M * Nn, dtype=torch.float32, device="cuda")
    Y64 = torch.empty(M * Nn, dtype=torch.float64, device="cuda")
    log = vt.alloc_log(M * Nn)
    ws = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, M, Nn, K, 1))
    vt.vt_conv2d_f64_round_log(vt.VT_CONV_FORWARD, d, Cout, Xd, Wd, None, Y32, Y64, 0, tau, log, ws)
    torch.cuda.synchronize()
    y64 = Y64.cpu().numpy().reshape(N, Ho, Wo, Cout)
    Xp = np.pad(X, ((0, 0), (pad, pad), (pad, pad), (0, 0)))
    wcol = np.linalg.norm(Wt.reshape(-1, Cout), axis=0)
    samples = [(0, 0, 0), (N - 1, Ho - 1, Wo - 1), (0, 0, Wo - 1), (N - 1, Ho - 1, 0)] + \
              [tuple(v) for v in g.integers(0, [N, Ho, Wo], (24, 3))]
    for n, ho, wo in samples:
        patch = Xp[n:n + 1, ho * stride: ho * stride + KH, wo * stride: wo * stride + KW, :]
        truth = vo.conv2d_fwd(patch, Wt, order=2)[0, 0, 0]                  # the oracle on the receptive field
        assert np.all(np.abs(y64[n, ho, wo] - truth) <= 1e-12 * np.linalg.norm(patch) * wcol + 1e-300), name
    _hook_parity(Y32.cpu().numpy(), y64, log, int(log.count.item()), tau)
    del Y64, Y32, log, ws
    # ---- weight gradient (split-K over the N Ho Wo output positions)
    dY = g.standard_normal((M, Cout)) * 1e-3
    dYd = torch.from_numpy(dY).cuda().reshape(-1)
    Mg, Ng, Kg = vt.vt_conv2d_gemm_shape(d, Cout, vt.VT_CONV_WEIGHT_GRAD)
    G32 = torch.empty(Mg * Ng, dtype=torch.float32, device="cuda")
    G64 = torch.empty(Mg * Ng, dtype=torch.float64, device="cuda")
    log = vt.alloc_log(Mg * Ng)
    ws = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, Mg, Ng, Kg, 1))
    vt.vt_conv2d_f64_round_log(vt.VT_CONV_WEIGHT_GRAD, d, Cout, Xd, dYd, None, G32, G64, 0, tau, log, ws)
    torch.cuda.synchronize()
    g64 = G64.cpu().numpy().reshape(KH, KW, Cin, Cout)
    for kh, kw, ci in [(0, 0, 0), (KH - 1, KW - 1, Cin - 1)] + [tuple(v) for v in g.integers(0, [KH, KW, Cin], (3, 3))]:
        col = Xp[:, kh: kh + (Ho - 1) * stride + 1: stride, kw: kw + (Wo - 1) * stride + 1: stride, ci].reshape(1, -1)
        truth = vo.gemm_f64(np.ascontiguousarray(col), dY, order=2)[0]      # the oracle's dot products over all positions
        assert np.all(np.abs(g64[kh, kw, ci] - truth) <= 1e-12 * np.linalg.norm(col) * np.linalg.norm(dY, axis=0) + 1e-300), name
    _hook_parity(G32.cpu().numpy(), g64, log, int(log.count.item()), tau)


@pytest.mark.parametrize("name,geom", [
    ("3x3 bottleneck", (64, 56, 56, 64, 3, 3, 64, 1, 1)),
    ("3x3/2 (one GEMM per stride phase)", (64, 56, 56, 128, 3, 3, 128, 2, 1)),
    ("1x1/2 downsample (one phase has taps)", (64, 56, 56, 256, 1, 1, 512, 2, 0)),
])
def test_resnet_input_gradients_full_size(name, geom):
    """The gradient with respect to the layer's input at batch 64: two whole images against the oracle's
    extended-precision loops, every output's FP32 value and the whole log against the oracle's hook."""
    import torch
    import paper_2403_09603_amd as vt
    N, H, W, Cin, KH, KW, Cout, stride, pad = geom
    g = si.rng(si.seed_for(4, 60) + Cin + KH)
    Wt = _f32grid(g.standard_normal((KH, KW, Cin, Cout)) * np.sqrt(2.0 / (KH * KW * Cin)))
    _, Ho, Wo = vo.conv2d_geometry((N, H, W, Cin), KH, KW, stride, pad, 1)
    dY = g.standard_normal((N, Ho, Wo, Cout))
    tau = 2.0 ** -5
    d = vt.Conv2d(N, H, W, Cin, KH, KW, stride, stride, pad, pad, 1, 1)
    M, Nn, K = vt.vt_conv2d_gemm_shape(d, Cout, vt.VT_CONV_DATA_GRAD)
    assert (M, Nn, K) == (N * H * W, Cin, KH * KW * Cout)
    dYd, Wd = torch.from_numpy(dY).cuda().reshape(-1), torch.from_numpy(Wt).cuda().reshape(-1)
    X32 = torch.empty(M * Nn, dtype=torch.float32, device="cuda")
    X64 = torch.empty(M * Nn, dtype=torch.float64, device="cuda")
    log = vt.alloc_log(M * Nn)
    ws = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_CONV_DGRAD_ROUND_LOG, M, Nn, K, 1))
    vt.vt_conv2d_f64_round_log(vt.VT_CONV_DATA_GRAD, d, Cout, dYd, Wd, None, X32, X64, 0, tau, log, ws)
    torch.cuda.synchronize()
    x64 = X64.cpu().numpy().reshape(N, H, W, Cin)
    wnorm = np.sqrt((Wt ** 2).sum(axis=(0, 1, 3)))                          # per input channel, over (kh, kw, co)
    for n in (0, N - 1):
        truth = vo.conv2d_dgrad(dY[n:n + 1], Wt, (1, H, W, Cin), stride=stride, pad=pad, order=2)[0]
        # squared norm of each input position's row of the gathered view: the dY positions that read it
        S = (dY[n] ** 2).sum(axis=2)
        rn2 = np.zeros((H, W))
        for kh in range(KH):
            for kw in range(KW):
                for ho in range(Ho):
                    h = ho * stride - pad + kh
                    if 0 <= h < H:
                        w = np.arange(Wo) * stride - pad + kw
                        ok = (w >= 0) & (w < W)
                        rn2[h, w[ok]] += S[ho, ok]
        bound = 1e-12 * np.sqrt(rn2)[:, :, None] * wnorm[None, None, :] + 1e-300
        assert np.all(np.abs(x64[n] - truth) <= bound), name
    _hook_parity(X32.cpu().numpy(), x64, log, int(log.count.item()), tau)

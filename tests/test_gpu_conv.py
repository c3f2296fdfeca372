"""GPU parity: convolution layers (forward, weight gradient, input gradient) through the implicit-im2col GEMM.

FP64 values within 1e-12 * ||patch|| ||filter column|| (+ |bias|) of the oracle's extended-precision
convolution (the definition written out as loops); FP32 outputs, index list, direction bits and
count bit-exact against the oracle's round/log of the kernel's own FP64 values.  The same layer run
as an explicit GEMM over a materialised im2col matrix must give the same FP64 bits (same plan, same
accumulation order).  Geometries follow the ResNet-50 layer types at reduced size.
"""
import numpy as np
import pytest

import synth_inputs as si
from oracle import vt_oracle as vo

pytestmark = pytest.mark.gpu

FWD, WGRAD, DGRAD = 0, 1, 2


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def _bits(y):
    return np.ascontiguousarray(y, np.float32).view(np.uint32)


def _pair(v):
    return (v, v) if np.isscalar(v) else tuple(v)


def _im2col(X, KH, KW, stride, pad, dil):
    """rows (n,ho,wo) x taps (kh,kw,ci) matrix, zeros in the padding (test-side, numpy)."""
    (sh, sw), (ph, pw), (dh, dw) = _pair(stride), _pair(pad), _pair(dil)
    N, H, W, Cin = X.shape
    Ho = (H + 2 * ph - dh * (KH - 1) - 1) // sh + 1
    Wo = (W + 2 * pw - dw * (KW - 1) - 1) // sw + 1
    Xp = np.pad(X, ((0, 0), (ph, ph), (pw, pw), (0, 0)))
    col = np.empty((N, Ho, Wo, KH, KW, Cin))
    for kh in range(KH):
        for kw in range(KW):
            col[:, :, :, kh, kw, :] = Xp[:, kh * dh: kh * dh + (Ho - 1) * sh + 1: sh,
                                         kw * dw: kw * dw + (Wo - 1) * sw + 1: sw, :]
    return col.reshape(N * Ho * Wo, KH * KW * Cin)


def _check_log(r, tau):
    yo, io, do, co = vo.round_log(r["C64"].ravel(), tau)
    assert r["count"] == co
    assert np.array_equal(_bits(r["C32"].ravel()), _bits(yo))
    assert np.array_equal(r["idx"], io)
    nw = (co + 31) // 32
    if co:
        a = np.unpackbits(r["dir"].view(np.uint8)[:4 * nw], bitorder="little")[:co]
        b = np.unpackbits(do.view(np.uint8)[:4 * nw], bitorder="little")[:co]
        assert np.array_equal(a, b)


def _check_layer(G, geom, *, tau=2.0 ** -5, misalign=False, seed=0, relu_input=True):
    N, H, W, Cin, KH, KW, Cout, stride, pad, dil = geom
    g = si.rng(si.seed_for(4, 10 + seed))
    X = g.standard_normal((N, H, W, Cin))
    if relu_input:
        X = np.maximum(X, 0.0)                                   # post-ReLU structure: half exact zeros
    X = X.astype(np.float32).astype(np.float64)
    Wt = (g.standard_normal((KH, KW, Cin, Cout)) * np.sqrt(2.0 / (KH * KW * Cin))).astype(np.float32).astype(np.float64)
    bias = g.standard_normal(Cout) * 0.1
    col = _im2col(X, KH, KW, stride, pad, dil)
    kw = dict(stride=stride, pad=pad, dil=dil)
    out = {}
    # ---- forward
    truth = vo.conv2d_fwd(X, Wt, bias=bias, order=2, **kw).reshape(-1, Cout)
    bound = 1e-12 * (np.linalg.norm(col, axis=1)[:, None] * np.linalg.norm(Wt.reshape(-1, Cout), axis=0)[None, :]
                     + np.abs(bias)[None, :]) + 1e-300
    for variant in (0, 1):
        r = G.gpu_conv(FWD, X, Wt, KH, KW, bias=bias, tau=tau, variant=variant, misalign=misalign, **kw)
        assert r["shape"] == (col.shape[0], Cout, col.shape[1])
        assert np.all(np.abs(r["C64"] - truth) <= bound), float(np.max(np.abs(r["C64"] - truth) / bound))
        _check_log(r, tau)
        e = G.gpu_gemm(col, Wt.reshape(-1, Cout), bias=bias, tau=tau, variant=variant)
        assert np.array_equal(e["C64"][0], r["C64"])             # materialised im2col: same bits
        out[("fwd", variant)] = r
    # ---- weight gradient
    dY = (g.standard_normal((col.shape[0], Cout)) * 1e-3)
    _, Ho, Wo = vo.conv2d_geometry(X.shape, KH, KW, stride, pad, dil)
    truth = vo.conv2d_wgrad(X, dY.reshape(N, Ho, Wo, Cout), KH, KW, order=2, **kw).reshape(-1, Cout)
    bound = 1e-12 * np.linalg.norm(col, axis=0)[:, None] * np.linalg.norm(dY, axis=0)[None, :] + 1e-300
    for variant in (0, 1):
        r = G.gpu_conv(WGRAD, X, dY, KH, KW, tau=tau, variant=variant, misalign=misalign, **kw)
        assert r["shape"] == (col.shape[1], Cout, col.shape[0])
        assert np.all(np.abs(r["C64"] - truth) <= bound), float(np.max(np.abs(r["C64"] - truth) / bound))
        _check_log(r, tau)
        # the materialised matrix gives the same bits when both runs accumulate in the same order, that is
        # when the plan (tile, split factor) of the implicit view equals that of a stored transposed matrix
        import paper_2403_09603_amd as vt
        plain = KH == 1 and KW == 1 and _pair(stride) == (1, 1) and _pair(pad) == (0, 0)
        layout = vt.VT_A_TRANSPOSED if plain else vt.VT_A_IM2COL_T
        if vt.vt_gemm_plan(col.shape[1], Cout, col.shape[0], 1, transA=layout) == \
                vt.vt_gemm_plan(col.shape[1], Cout, col.shape[0], 1, transA=True):
            e = G.gpu_gemm(col, dY, transA=True, tau=tau, variant=variant)
            assert np.array_equal(e["C64"][0], r["C64"])
        out[("wgrad", variant)] = r
    # ---- input gradient
    dYn = dY.reshape(N, Ho, Wo, Cout) * 1e3
    truth = vo.conv2d_dgrad(dYn, Wt, X.shape, order=2, **kw).reshape(-1, Cin)
    # the gathered matrix of the output gradient, built test-side by scattering (n, ho, wo, kh, kw) -> input position
    (sh, sw), (ph, pw), (dh, dw) = _pair(stride), _pair(pad), _pair(dil)
    view = np.zeros((N, H, W, KH, KW, Cout))
    for kh in range(KH):
        for kw_ in range(KW):
            for ho in range(Ho):
                h = ho * sh - ph + kh * dh
                if not 0 <= h < H:
                    continue
                for wo in range(Wo):
                    w = wo * sw - pw + kw_ * dw
                    if 0 <= w < W:
                        view[:, h, w, kh, kw_, :] = dYn[:, ho, wo, :]
    view = view.reshape(N * H * W, KH * KW * Cout)
    Wp = np.ascontiguousarray(Wt.transpose(0, 1, 3, 2)).reshape(KH * KW * Cout, Cin)
    bound = 1e-12 * np.linalg.norm(view, axis=1)[:, None] * np.linalg.norm(Wp, axis=0)[None, :] + 1e-300
    for variant in (0, 1):
        r = G.gpu_conv(DGRAD, dYn, Wt, KH, KW, tau=tau, variant=variant, misalign=misalign, xshape=X.shape, **kw)
        assert r["shape"] == (N * H * W, Cin, KH * KW * Cout)
        assert np.all(np.abs(r["C64"] - truth) <= bound), float(np.max(np.abs(r["C64"] - truth) / bound))
        _check_log(r, tau)
        one_gemm_over_the_view = not (KH == 1 and KW == 1 and _pair(stride) == (1, 1) and _pair(pad) == (0, 0)) and \
            (_pair(stride) == (1, 1) or max(_pair(stride)) > 2 or Cin % 2 == 1)
        if one_gemm_over_the_view:      # (strided layers with even C run one GEMM per stride phase instead)
            e = G.gpu_gemm(view, Wp, tau=tau, variant=variant)
            assert np.array_equal(e["C64"][0], r["C64"])         # materialised view: same bits
        out[("dgrad", variant)] = r
    return out


SMALL = [  # (N, H, W, C, KH, KW, Cout, stride, pad, dil)
    (2, 9, 11, 3, 3, 3, 4, 1, 1, 1),
    (1, 12, 10, 2, 7, 7, 3, 2, 3, 1),
    (2, 8, 7, 4, 1, 1, 5, 2, 0, 1),
    (1, 10, 13, 3, 3, 2, 2, (2, 1), (1, 0), (1, 2)),
    (1, 9, 9, 2, 3, 3, 2, 1, 2, 2),
    (1, 4, 4, 1, 5, 5, 1, 1, 2, 1),
    (2, 9, 7, 5, 1, 1, 6, 1, 0, 1),          # 1 x 1 at every position, odd channel count: the plain-matrix route
    (3, 20, 17, 64, 1, 1, 70, 1, 0, 3),      # the same with whole tiles, a ragged edge, and a dilation that cannot matter
    (1, 11, 10, 4, 3, 3, 6, 3, 1, 1),        # stride 3: the input gradient as one GEMM over the strided view
    (2, 10, 13, 4, 3, 2, 2, (2, 1), (1, 0), (1, 2)),   # stride phases along one axis only, dilation along the other
    (1, 9, 12, 6, 4, 3, 4, 2, (0, 2), (2, 1)),         # dilation equal to the stride: one phase gets every filter row
]


@pytest.mark.parametrize("geom", SMALL)
def test_small_geometries(G, geom):
    _check_layer(G, geom)


@pytest.mark.parametrize("geom,name", [
    ((2, 34, 30, 3, 7, 7, 64, 2, 3, 1), "first convolution 7x7/2, 3 channels (odd: scalar loads)"),
    ((2, 28, 28, 64, 3, 3, 64, 1, 1, 1), "3x3 bottleneck, taps 576"),
    ((2, 28, 28, 64, 1, 1, 256, 1, 0, 1), "1x1 expand"),
    ((2, 28, 28, 128, 3, 3, 128, 2, 1, 1), "3x3 stride 2"),
    ((3, 28, 28, 256, 1, 1, 512, 2, 0, 1), "1x1 stride 2 downsample"),
    ((1, 21, 19, 6, 3, 3, 70, 1, 1, 2), "ragged everything, dilation 2"),
])
def test_resnet_layer_types(G, geom, name):
    _check_layer(G, geom, seed=1)


def test_image_on_an_8_byte_boundary_uses_scalar_loads(G):
    _check_layer(G, (2, 14, 14, 32, 3, 3, 64, 1, 1, 1), misalign=True, seed=2)


def test_weight_gradient_with_split_k_is_deterministic(G):
    import paper_2403_09603_amd as vt
    geom = (4, 48, 48, 16, 3, 3, 32, 1, 1, 1)
    N, H, W, Cin, KH, KW, Cout, stride, pad, dil = geom
    assert vt.vt_gemm_plan(KH * KW * Cin, Cout, N * H * W, 1, transA=vt.VT_A_IM2COL_T)[2] > 1
    a = _check_layer(G, geom, seed=3)
    b = _check_layer(G, geom, seed=3)
    for key in a:
        assert np.array_equal(a[key]["C64"], b[key]["C64"]) and np.array_equal(a[key]["idx"], b[key]["idx"])
    assert (a[("wgrad", 0)]["C64"] != a[("wgrad", 1)]["C64"]).mean() > 0.3


@pytest.mark.parametrize("geom", [(2, 13, 12, 8, 3, 3, 16, 2, 1, 1), (2, 12, 12, 6, 3, 3, 10, 1, 1, 1)])
def test_packed_log_from_every_mode(G, geom):
    """Forward, weight gradient and input gradient (per stride phase and as one GEMM) writing the
    packed ternary log: bytes, FP32 outputs and count against the oracle on the kernel's FP64 values;
    the input gradient's values must not depend on the log format."""
    N, H, W, Cin, KH, KW, Cout, stride, pad, dil = geom
    g = si.rng(si.seed_for(4, 30))
    X = np.maximum(g.standard_normal((N, H, W, Cin)), 0.0)
    Wt = g.standard_normal((KH, KW, Cin, Cout)) * 0.2
    _, Ho, Wo = vo.conv2d_geometry(X.shape, KH, KW, stride, pad, dil)
    dY = g.standard_normal((N, Ho, Wo, Cout))
    kw = dict(stride=stride, pad=pad, dil=dil)
    tau = 0.25
    for mode, a, b, extra in ((FWD, X, Wt, {}), (WGRAD, X, dY, {}), (DGRAD, dY, Wt, {"xshape": X.shape})):
        for variant in (0, 1):
            r = G.gpu_conv(mode, a, b, KH, KW, tau=tau, variant=variant, dense=True, **kw, **extra)
            yo, to, co = vo.round_log_dense(r["C64"].ravel(), tau)
            assert r["count"] == co and co > r["C64"].size // 3
            assert np.array_equal(_bits(r["C32"].ravel()), _bits(yo)) and np.array_equal(r["tlog"], to)
            if mode == DGRAD:
                sparse = G.gpu_conv(mode, a, b, KH, KW, tau=tau, variant=variant, **kw, **extra)
                assert np.array_equal(sparse["C64"], r["C64"])


def test_empty_and_degenerate_layers(G):
    g = si.rng(si.seed_for(4, 20))
    X = g.standard_normal((1, 2, 9, 3))
    r = G.gpu_conv(FWD, X, g.standard_normal((3, 3, 3, 4)), 3, 3)          # kernel does not fit: no outputs
    assert r["count"] == 0 and r["shape"][0] == 0
    r = G.gpu_conv(WGRAD, X, np.zeros((1, 0, 7, 4)), 3, 3, tau=0.25)       # no positions: gradient is zero
    assert r["shape"] == (27, 4, 0) and np.array_equal(r["C64"], np.zeros((27, 4))) and r["count"] == 0
    r = G.gpu_conv(DGRAD, np.zeros((1, 0, 7, 4)), g.standard_normal((3, 3, 3, 4)), 3, 3, tau=0.25, xshape=(1, 2, 9, 3))
    assert r["shape"] == (18, 3, 36) and np.array_equal(r["C64"], np.zeros((18, 3))) and r["count"] == 0   # no outputs: zero gradient
    r = G.gpu_conv(DGRAD, np.zeros((2, 3, 3, 0)), np.zeros((3, 3, 5, 0)), 3, 3, pad=1, xshape=(2, 3, 3, 5))  # no output channels
    assert r["shape"] == (18, 5, 0) and np.array_equal(r["C64"], np.zeros((18, 5))) and r["count"] == 0

"""Pins for the oracle's convolution layer (forward, weight gradient and input gradient).

The oracle writes the definition out as nested loops over channels-last arrays.  It is pinned
here against things that are not itself: library routines (scipy's 2-D correlation, PyTorch's
CPU convolution and its autograd), exact integer brute force in pure Python, the reduction of a
1x1 convolution to a matrix product, the adjoint identity between the forward map and the weight
gradient and between the forward map and the input gradient (a scatter over output positions
where the oracle gathers over input positions), the closed-form output sizes of the ResNet-50 geometry, and the stated summation order
(re-accumulated for sampled outputs with Python floats).
"""
import itertools

import numpy as np
import pytest

import synth_inputs as si
from oracle import vt_oracle as vo

GEOMS = [  # (N, H, W, C, KH, KW, Cout, stride, pad, dil)
    (2, 9, 11, 3, 3, 3, 4, 1, 1, 1),
    (1, 12, 10, 2, 7, 7, 3, 2, 3, 1),            # first ResNet convolution, scaled down
    (2, 8, 7, 4, 1, 1, 5, 2, 0, 1),              # strided 1x1 (downsample)
    (1, 10, 13, 3, 3, 2, 2, (2, 1), (1, 0), (1, 2)),   # everything asymmetric
    (1, 9, 9, 2, 3, 3, 2, 1, 2, 2),              # dilation
    (1, 4, 4, 1, 5, 5, 1, 1, 2, 1),              # kernel larger than the image
]


def _pair(v):
    return (v, v) if np.isscalar(v) else tuple(v)


def _rand(shape, seed):
    return si.rng(seed).standard_normal(shape)


def test_output_sizes_of_the_resnet_geometry():
    for (H, K, s, p, want) in [(224, 7, 2, 3, 112), (56, 3, 1, 1, 56), (56, 1, 1, 0, 56), (56, 3, 2, 1, 28),
                               (56, 1, 2, 0, 28), (14, 3, 2, 1, 7), (7, 3, 1, 1, 7)]:
        _, Ho, Wo = vo.conv2d_geometry((1, H, H, 1), K, K, s, p, 1)
        assert (Ho, Wo) == (want, want)
    _, Ho, Wo = vo.conv2d_geometry((1, 2, 9, 1), 3, 3, 1, 0, 1)       # kernel does not fit: empty output
    assert Ho == 0 and Wo == 7


@pytest.mark.parametrize("geom", GEOMS)
def test_forward_and_weight_gradient_against_pytorch(geom):
    torch = pytest.importorskip("torch")
    N, H, W, Cin, KH, KW, Cout, stride, pad, dil = geom
    X, Wt, b = _rand((N, H, W, Cin), 11), _rand((KH, KW, Cin, Cout), 12), _rand(Cout, 13)
    xt = torch.from_numpy(X).permute(0, 3, 1, 2)
    wt = torch.from_numpy(Wt).permute(3, 2, 0, 1).clone().requires_grad_(True)
    yt = torch.nn.functional.conv2d(xt, wt, torch.from_numpy(b), stride=_pair(stride), padding=_pair(pad),
                                    dilation=_pair(dil))
    want = yt.detach().permute(0, 2, 3, 1).numpy()
    for order in (0, 1, 2):
        got = vo.conv2d_fwd(X, Wt, stride=stride, pad=pad, dil=dil, bias=b, order=order)
        assert got.shape == want.shape
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-12 * KH * KW * Cin)
    dY = _rand(want.shape, 14)
    (yt * torch.from_numpy(dY).permute(0, 3, 1, 2)).sum().backward()
    want_dw = wt.grad.permute(2, 3, 1, 0).numpy()
    for order in (0, 1, 2):
        got = vo.conv2d_wgrad(X, dY, KH, KW, stride=stride, pad=pad, dil=dil, order=order)
        np.testing.assert_allclose(got, want_dw, rtol=0, atol=1e-12 * max(dY[..., 0].size, 1))


def test_forward_against_scipy_correlation():
    sig = pytest.importorskip("scipy.signal")
    N, H, W, Cin, KH, KW, Cout, ph, pw = 2, 9, 12, 3, 3, 5, 2, 1, 2
    X, Wt = _rand((N, H, W, Cin), 21), _rand((KH, KW, Cin, Cout), 22)
    got = vo.conv2d_fwd(X, Wt, pad=(ph, pw), order=2)
    Xp = np.pad(X, ((0, 0), (ph, ph), (pw, pw), (0, 0)))
    for n, co in itertools.product(range(N), range(Cout)):
        want = sum(sig.correlate2d(Xp[n, :, :, ci], Wt[:, :, ci, co], mode="valid") for ci in range(Cin))
        np.testing.assert_allclose(got[n, :, :, co], want, rtol=0, atol=1e-12)


def _brute(X, Wt, stride, pad, dil):
    """Exact integer convolution and weight gradient of an all-ones dY, pure Python."""
    (sh, sw), (ph, pw), (dh, dw) = _pair(stride), _pair(pad), _pair(dil)
    N, H, W, Cin = X.shape
    KH, KW, _, Cout = Wt.shape
    Ho = (H + 2 * ph - dh * (KH - 1) - 1) // sh + 1
    Wo = (W + 2 * pw - dw * (KW - 1) - 1) // sw + 1
    Y = np.zeros((N, Ho, Wo, Cout), dtype=object)
    for n, ho, wo, co, kh, kw, ci in itertools.product(range(N), range(Ho), range(Wo), range(Cout), range(KH),
                                                       range(KW), range(Cin)):
        h, w = ho * sh - ph + kh * dh, wo * sw - pw + kw * dw
        if 0 <= h < H and 0 <= w < W:
            Y[n, ho, wo, co] += int(X[n, h, w, ci]) * int(Wt[kh, kw, ci, co])
    return Y


@pytest.mark.parametrize("geom", GEOMS)
def test_integer_data_is_exact_against_brute_force(geom):
    N, H, W, Cin, KH, KW, Cout, stride, pad, dil = geom
    g = si.rng(31)
    X = g.integers(-9, 10, (N, H, W, Cin)).astype(np.float64)
    Wt = g.integers(-9, 10, (KH, KW, Cin, Cout)).astype(np.float64)
    want = _brute(X, Wt, stride, pad, dil)
    for order in (0, 1, 2):
        got = vo.conv2d_fwd(X, Wt, stride=stride, pad=pad, dil=dil, order=order)
        assert got.shape == want.shape and np.array_equal(got, want.astype(np.float64))
    # adjoint identity, exact on integers: <conv(X, W), dY> = <W, wgrad(X, dY)>
    dY = g.integers(-9, 10, want.shape).astype(np.float64)
    lhs = int(sum(int(a) * int(b) for a, b in zip(want.ravel(), dY.ravel())))
    for order in (0, 1, 2):
        dW = vo.conv2d_wgrad(X, dY, KH, KW, stride=stride, pad=pad, dil=dil, order=order)
        assert int(sum(int(a) * int(b) for a, b in zip(dW.ravel(), Wt.ravel()))) == lhs
        # each weight-gradient entry is the forward map of a one-hot weight tensor contracted with dY
        for (kh, kw, ci, co) in [(0, 0, 0, 0), (KH - 1, KW - 1, Cin - 1, Cout - 1), (KH // 2, 0, Cin - 1, 0)]:
            E = np.zeros_like(Wt)
            E[kh, kw, ci, co] = 1.0
            assert dW[kh, kw, ci, co] == float((_brute(X, E, stride, pad, dil) * dY.astype(object)).sum())


def test_1x1_strided_convolution_is_a_matrix_product():
    X, Wt = _rand((2, 8, 6, 5), 41), _rand((1, 1, 5, 7), 42)
    b = _rand(7, 43)
    rows = X[:, ::2, ::2, :].reshape(-1, 5)
    for order in (0, 1):
        got = vo.conv2d_fwd(X, Wt, stride=2, bias=b, order=order)
        want = vo.gemm_f64(rows, Wt.reshape(5, 7), bias=b, order=order)
        assert np.array_equal(got.reshape(-1, 7), want)                 # same terms in the same order
        np.testing.assert_allclose(got.reshape(-1, 7), rows @ Wt.reshape(5, 7) + b, rtol=0, atol=1e-13)
    dY = _rand((2, 4, 3, 7), 44)
    for order in (0, 1):
        got = vo.conv2d_wgrad(X, dY, 1, 1, stride=2, order=order)
        want = vo.gemm_f64(rows, dY.reshape(-1, 7), transA=True, order=order)
        assert np.array_equal(got.reshape(5, 7), want)


def test_summation_order_is_the_stated_one():
    """order 0 adds the taps in ascending (kh, kw, ci), order 1 in descending order; the weight
    gradient adds output positions in ascending / descending (n, ho, wo)."""
    N, H, W, Cin, KH, KW, Cout = 2, 6, 7, 3, 3, 2, 2
    X, Wt = _rand((N, H, W, Cin), 51), _rand((KH, KW, Cin, Cout), 52)
    ph, pw = 1, 1
    Y0 = vo.conv2d_fwd(X, Wt, pad=(ph, pw), order=0)
    Y1 = vo.conv2d_fwd(X, Wt, pad=(ph, pw), order=1)
    assert (Y0 != Y1).any()
    Ho, Wo = Y0.shape[1:3]
    taps = list(itertools.product(range(KH), range(KW), range(Cin)))
    for (n, ho, wo, co) in [(0, 0, 0, 0), (1, Ho - 1, Wo - 1, 1), (1, 2, 3, 0)]:
        for order, seq in ((0, taps), (1, taps[::-1])):
            acc = 0.0
            for kh, kw, ci in seq:
                h, w = ho - ph + kh, wo - pw + kw
                x = float(X[n, h, w, ci]) if 0 <= h < H and 0 <= w < W else 0.0
                acc = acc + x * float(Wt[kh, kw, ci, co])
            assert acc == (Y0, Y1)[order][n, ho, wo, co]
    dY = _rand(Y0.shape, 53)
    pos = list(itertools.product(range(N), range(Ho), range(Wo)))
    for order, seq in ((0, pos), (1, pos[::-1])):
        dW = vo.conv2d_wgrad(X, dY, KH, KW, pad=(ph, pw), order=order)
        for (kh, kw, ci, co) in [(0, 0, 0, 0), (2, 1, 2, 1)]:
            acc = 0.0
            for n, ho, wo in seq:
                h, w = ho - ph + kh, wo - pw + kw
                x = float(X[n, h, w, ci]) if 0 <= h < H and 0 <= w < W else 0.0
                acc = acc + x * float(dY[n, ho, wo, co])
            assert acc == dW[kh, kw, ci, co]


def _brute_dgrad(dY, Wt, xshape, stride, pad, dil):
    """Exact integer input gradient by scattering every (output position, tap) product, pure Python."""
    (sh, sw), (ph, pw), (dh, dw) = _pair(stride), _pair(pad), _pair(dil)
    N, H, W, Cin = xshape
    KH, KW, _, Cout = Wt.shape
    _, Ho, Wo, _ = dY.shape
    dX = np.zeros(xshape, dtype=object)
    for n, ho, wo, co, kh, kw, ci in itertools.product(range(N), range(Ho), range(Wo), range(Cout), range(KH),
                                                       range(KW), range(Cin)):
        h, w = ho * sh - ph + kh * dh, wo * sw - pw + kw * dw
        if 0 <= h < H and 0 <= w < W:
            dX[n, h, w, ci] += int(dY[n, ho, wo, co]) * int(Wt[kh, kw, ci, co])
    return dX


@pytest.mark.parametrize("geom", GEOMS)
def test_input_gradient_against_pytorch(geom):
    torch = pytest.importorskip("torch")
    N, H, W, Cin, KH, KW, Cout, stride, pad, dil = geom
    X, Wt = _rand((N, H, W, Cin), 61), _rand((KH, KW, Cin, Cout), 62)
    xt = torch.from_numpy(X).permute(0, 3, 1, 2).clone().requires_grad_(True)
    wt = torch.from_numpy(Wt).permute(3, 2, 0, 1).clone()
    yt = torch.nn.functional.conv2d(xt, wt, None, stride=_pair(stride), padding=_pair(pad), dilation=_pair(dil))
    dY = _rand(tuple(yt.permute(0, 2, 3, 1).shape), 63)
    (yt * torch.from_numpy(dY).permute(0, 3, 1, 2)).sum().backward()
    want = xt.grad.permute(0, 2, 3, 1).numpy()
    for order in (0, 1, 2):
        got = vo.conv2d_dgrad(dY, Wt, X.shape, stride=stride, pad=pad, dil=dil, order=order)
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-12 * KH * KW * Cout)


@pytest.mark.parametrize("geom", GEOMS)
def test_input_gradient_on_integers_is_exact(geom):
    N, H, W, Cin, KH, KW, Cout, stride, pad, dil = geom
    g = si.rng(71)
    X = g.integers(-9, 10, (N, H, W, Cin)).astype(np.float64)
    Wt = g.integers(-9, 10, (KH, KW, Cin, Cout)).astype(np.float64)
    Y = _brute(X, Wt, stride, pad, dil)
    dY = g.integers(-9, 10, Y.shape).astype(np.float64)
    want = _brute_dgrad(dY, Wt, X.shape, stride, pad, dil)
    lhs = int(sum(int(a) * int(b) for a, b in zip(Y.ravel(), dY.ravel())))
    for order in (0, 1, 2):
        got = vo.conv2d_dgrad(dY, Wt, X.shape, stride=stride, pad=pad, dil=dil, order=order)
        assert np.array_equal(got, want.astype(np.float64))
        # adjoint identity, exact on integers: <conv(X, W), dY> = <X, dgrad(dY, W)>
        assert int(sum(int(a) * int(b) for a, b in zip(got.ravel(), X.ravel()))) == lhs


def test_input_gradient_of_a_1x1_convolution_is_a_matrix_product():
    Wt = _rand((1, 1, 5, 7), 81)
    dY = _rand((2, 4, 3, 7), 82)
    for order in (0, 1):
        got = vo.conv2d_dgrad(dY, Wt, (2, 8, 6, 5), stride=2, order=order)
        want = vo.gemm_f64(dY.reshape(-1, 7), Wt.reshape(5, 7), transB=True, order=order)
        assert np.array_equal(got[:, ::2, ::2, :].reshape(-1, 5), want)     # same terms in the same order
        mask = np.ones((8, 6), bool)
        mask[::2, ::2] = False
        assert not got[:, mask, :].any()                                    # positions no output reads
    got = vo.conv2d_dgrad(dY, Wt, (2, 4, 3, 5), order=0)                    # stride 1: every position
    assert np.array_equal(got.reshape(-1, 5), vo.gemm_f64(dY.reshape(-1, 7), Wt.reshape(5, 7), transB=True, order=0))


def test_input_gradient_summation_order_is_the_stated_one():
    """order 0 adds the terms in ascending (kh, kw, co), order 1 in descending order."""
    N, H, W, Cin, KH, KW, Cout, s, p = 1, 7, 6, 2, 3, 3, 3, 2, 1
    Wt = _rand((KH, KW, Cin, Cout), 91)
    _, Ho, Wo = vo.conv2d_geometry((N, H, W, Cin), KH, KW, s, p, 1)
    dY = _rand((N, Ho, Wo, Cout), 92)
    D0 = vo.conv2d_dgrad(dY, Wt, (N, H, W, Cin), stride=s, pad=p, order=0)
    D1 = vo.conv2d_dgrad(dY, Wt, (N, H, W, Cin), stride=s, pad=p, order=1)
    assert (D0 != D1).any()
    terms = list(itertools.product(range(KH), range(KW), range(Cout)))
    for (h, w, ci) in [(0, 0, 0), (H - 1, W - 1, 1), (3, 2, 0), (2, 3, 1)]:
        for order, seq in ((0, terms), (1, terms[::-1])):
            acc = 0.0
            for kh, kw, co in seq:
                hs, ws = h + p - kh, w + p - kw
                ok = hs >= 0 and ws >= 0 and hs % s == 0 and ws % s == 0 and hs // s < Ho and ws // s < Wo
                g = float(dY[0, hs // s, ws // s, co]) if ok else 0.0
                acc = acc + g * float(Wt[kh, kw, ci, co])
            assert acc == (D0, D1)[order][0, h, w, ci]


def test_invalid_geometry_is_rejected():
    with pytest.raises(ValueError):
        vo.conv2d_geometry((1, 4, 4, 1), 0, 3)
    with pytest.raises(ValueError):
        vo.conv2d_geometry((1, 4, 4, 1), 3, 3, stride=0)

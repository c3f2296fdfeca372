"""Pins for the oracle's element-wise and row-wise layers (residual add, ReLU, GELU, layer norm,
softmax): PyTorch's CPU implementations in float64 (library routines), closed forms and identities,
and the stated summation order re-accumulated with Python floats."""
import math

import numpy as np
import pytest

import synth_inputs as si
from oracle import vt_oracle as vo

torch = pytest.importorskip("torch")
F = torch.nn.functional


def _x(shape, seed, scale=1.0):
    return si.rng(si.seed_for(9, seed)).standard_normal(shape) * scale


def test_elementwise_against_pytorch_and_identities():
    x = np.concatenate([_x(5000, 1, 3.0), [0.0, -0.0, 1e-300, -1e-300, 40.0, -40.0, 1e6, -1e6]])
    b = _x(x.size, 2)
    t = torch.from_numpy(x)
    for exact in (False, True):
        assert np.array_equal(vo.elementwise(vo.EW_ADD, x, b, exact=exact), x + b)       # one exact-rounded addition
        np.testing.assert_array_equal(vo.elementwise(vo.EW_RELU, x, exact=exact), F.relu(t).numpy())
        np.testing.assert_allclose(vo.elementwise(vo.EW_GELU_TANH, x, exact=exact), F.gelu(t, approximate="tanh").numpy(),
                                   rtol=0, atol=4e-16 * np.maximum(np.abs(x), 1.0).max())
        np.testing.assert_allclose(vo.elementwise(vo.EW_GELU_ERF, x, exact=exact), F.gelu(t).numpy(),
                                   rtol=0, atol=4e-16 * np.maximum(np.abs(x), 1.0).max())
    g = vo.elementwise(vo.EW_GELU_ERF, x, exact=True)
    np.testing.assert_allclose(g - vo.elementwise(vo.EW_GELU_ERF, -x, exact=True), x, rtol=1e-15, atol=1e-300)  # odd part is x/2
    assert vo.elementwise(vo.EW_GELU_TANH, np.zeros(1))[0] == 0.0
    assert vo.elementwise(vo.EW_GELU_TANH, np.array([40.0]))[0] == 40.0 and vo.elementwise(vo.EW_GELU_ERF, np.array([-40.0]))[0] == 0.0
    assert math.isnan(vo.elementwise(vo.EW_RELU, np.array([np.nan]))[0])
    assert math.copysign(1.0, vo.elementwise(vo.EW_RELU, np.array([-0.0]))[0]) == 1.0


@pytest.mark.parametrize("rows,cols", [(1, 1), (3, 7), (5, 768), (2, 1025)])
def test_layernorm_against_pytorch_and_summation_order(rows, cols):
    x = _x((rows, cols), 10 + cols, 2.0) + 0.3
    gamma, beta = _x(cols, 11) + 1.0, _x(cols, 12)
    want = F.layer_norm(torch.from_numpy(x), (cols,), torch.from_numpy(gamma), torch.from_numpy(beta), 1e-5).numpy()
    for order in (0, 1, 2):
        np.testing.assert_allclose(vo.layernorm(x, gamma, beta, 1e-5, order), want, rtol=0, atol=1e-13 * np.abs(want).max() + 1e-13)
    plain = vo.layernorm(x, eps=0.0, order=2)
    if cols > 1:
        np.testing.assert_allclose(plain.mean(axis=1), 0.0, atol=1e-14)
        np.testing.assert_allclose((plain ** 2).mean(axis=1), 1.0, atol=1e-13)          # unit biased variance
    # the stated order, for one row, with Python floats
    for order in (0, 1):
        seq = list(range(cols)) if order == 0 else list(range(cols - 1, -1, -1))
        s = 0.0
        for c in seq:
            s = s + float(x[0, c])
        mean = s / cols
        q = 0.0
        for c in seq:
            d = float(x[0, c]) - mean
            q = q + d * d
        rstd = 1.0 / math.sqrt(q / cols + 1e-5)
        got = vo.layernorm(x, gamma, beta, 1e-5, order)[0]
        for c in (0, cols // 2, cols - 1):
            assert got[c] == (float(x[0, c]) - mean) * rstd * float(gamma[c]) + float(beta[c])


@pytest.mark.parametrize("rows,cols,period", [(4, 9, 0), (12, 6, 6), (7, 1024, 0), (10, 5, 5), (6, 8, 3)])
def test_softmax_against_pytorch_and_structure(rows, cols, period):
    x = _x((rows, cols), 20 + cols, 4.0)
    scale = 0.125
    z = torch.from_numpy(x) * scale
    if period:
        seen = (torch.arange(rows) % period + 1).clamp(max=cols)
        mask = torch.arange(cols)[None, :] < seen[:, None]
        z = z.masked_fill(~mask, float("-inf"))
    want = torch.softmax(z, dim=-1).numpy()
    for order in (0, 1, 2):
        got = vo.softmax(x, scale, period, order)
        np.testing.assert_allclose(got, want, rtol=0, atol=2e-16 * cols + 1e-16)
        np.testing.assert_allclose(got.sum(axis=1), 1.0, atol=1e-14)
        if period:
            assert np.all(got[~mask.numpy()] == 0.0) and np.all(got[mask.numpy()] > 0.0)
    # shift invariance (exact in long double up to its rounding) and the order of the sum
    np.testing.assert_allclose(vo.softmax(x + 3.0, scale, period, 2), vo.softmax(x, scale, period, 2), rtol=1e-14)
    r = rows - 1
    seen_r = min(r % period + 1, cols) if period else cols
    m = max(scale * float(v) for v in x[r, :seen_r])
    for order in (0, 1):
        seq = list(range(seen_r)) if order == 0 else list(range(seen_r - 1, -1, -1))
        s = 0.0
        for c in seq:
            s = s + math.exp(scale * float(x[r, c]) - m)
        got = vo.softmax(x, scale, period, order)[r]
        assert got[0] == math.exp(scale * float(x[r, 0]) - m) * (1.0 / s)


@pytest.mark.parametrize("rows,cols", [(2, 1), (9, 3), (640, 64), (1000, 7)])
def test_batchnorm_against_pytorch_and_summation_order(rows, cols):
    x = _x((rows, cols), 30 + cols, 2.0) + 0.5
    gamma, beta = _x(cols, 31) + 1.0, _x(cols, 32)
    xt = torch.from_numpy(x.T.copy()).reshape(1, cols, rows)                      # (N, C, L): statistics over N and L
    want = F.batch_norm(xt, None, None, torch.from_numpy(gamma), torch.from_numpy(beta), True, 0.0, 1e-5)
    want = want.reshape(cols, rows).T.numpy()
    for order in (0, 1, 2):
        got = vo.batchnorm(x, gamma, beta, 1e-5, order=order)
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-12 * (np.abs(want).max() + 1.0))
        np.testing.assert_array_equal(vo.batchnorm(x, gamma, beta, 1e-5, relu=True, order=order), np.maximum(got, 0.0))
    plain = vo.batchnorm(x, eps=0.0, order=2)
    if rows > 1:
        np.testing.assert_allclose(plain.mean(axis=0), 0.0, atol=1e-13)
        np.testing.assert_allclose((plain ** 2).mean(axis=0), 1.0, atol=1e-12)
    for order in (0, 1):                                                          # the stated order, one channel
        seq = list(range(rows)) if order == 0 else list(range(rows - 1, -1, -1))
        c = cols - 1
        s = 0.0
        for r in seq:
            s = s + float(x[r, c])
        mean = s / rows
        q = 0.0
        for r in seq:
            d = float(x[r, c]) - mean
            q = q + d * d
        rstd = 1.0 / math.sqrt(q / rows + 1e-5)
        got = vo.batchnorm(x, gamma, beta, 1e-5, order=order)
        for r in (0, rows // 2, rows - 1):
            assert got[r, c] == (float(x[r, c]) - mean) * rstd * float(gamma[c]) + float(beta[c])


def test_invalid_arguments():
    with pytest.raises(ValueError):
        vo.elementwise(7, np.ones(3))
    with pytest.raises(ValueError):
        vo.elementwise(vo.EW_ADD, np.ones(3))
    with pytest.raises(ValueError):
        vo.softmax(np.ones((2, 2)), causal_period=-1)

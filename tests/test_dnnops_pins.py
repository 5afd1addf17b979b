"""Pins of the Mish / layer-normalisation / softmax oracle against things other than itself."""
import math

import numpy as np
import pytest

from oracle import dnnops as orc

RNG = np.random.default_rng(4321)


# ---------------------------------------------------------------- Mish -------

def test_mish_special_values():
    assert orc.mish(0.0) == 0.0
    # mish'(0) = tanh(ln 2) = 3/5 exactly ((4-1)/(4+1))
    assert abs(orc.mish_grad(0.0) - 0.6) < 1e-15
    assert abs(orc.mish(1.0) - math.tanh(math.log(1.0 + math.e))) < 1e-15
    # x -> +inf: mish(x) -> x, mish'(x) -> 1;  x -> -inf: both -> 0 (like x*e^x)
    assert abs(orc.mish(40.0) - 40.0) < 1e-12 and abs(orc.mish_grad(40.0) - 1.0) < 1e-12
    assert abs(orc.mish(-40.0)) < 1e-15 and abs(orc.mish_grad(-40.0)) < 1e-15
    assert abs(orc.mish(-30.0) / (-30.0 * math.exp(-30.0)) - 1.0) < 1e-9
    # tanh(softplus(x)) = ((1+e^x)^2 - 1) / ((1+e^x)^2 + 1), a second route to the same value
    for x in (-3.0, -0.5, 0.25, 2.0, 7.0):
        u = (1.0 + math.exp(x)) ** 2
        assert abs(orc.mish(x) - x * (u - 1.0) / (u + 1.0)) < 1e-14


def test_mish_minimum_and_finite_differences():
    # the single minimum of mish lies near -1.1924 with value near -0.30884
    lo, hi = -2.0, -1.0
    for _ in range(80):
        mid = 0.5 * (lo + hi)
        if orc.mish_grad(mid) < 0:
            lo = mid
        else:
            hi = mid
    assert abs(lo - (-1.1924)) < 1e-3 and abs(orc.mish(lo) - (-0.30884)) < 1e-4
    x = RNG.standard_normal(200) * 3
    h = 1e-6
    fd = (orc.mish_fwd(x + h) - orc.mish_fwd(x - h)) / (2 * h)
    assert np.allclose(orc.mish_bwd(x, np.ones_like(x)), fd, rtol=1e-8, atol=1e-9)


def test_mish_vs_pytorch_fp64():
    import torch
    import torch.nn.functional as F
    x = torch.tensor(RNG.standard_normal((7, 33)) * 4, requires_grad=True)
    dy = RNG.standard_normal((7, 33))
    y = F.mish(x)
    y.backward(torch.tensor(dy))
    assert np.allclose(orc.mish_fwd(x.detach().numpy()), y.detach().numpy(), rtol=1e-13, atol=1e-14)
    assert np.allclose(orc.mish_bwd(x.detach().numpy(), dy), x.grad.numpy(), rtol=1e-12, atol=1e-13)


# ------------------------------------------------------ layer normalisation --

def test_layernorm_row_invariants():
    x = RNG.standard_normal((5, 37)) * 2 + 1
    eps = 1e-5
    y, mean, rstd = orc.layernorm_fwd(x, np.ones(37), np.zeros(37), eps)
    assert np.allclose(mean, x.mean(axis=1), atol=1e-14)
    assert np.allclose(rstd, 1 / np.sqrt(x.var(axis=1) + eps), rtol=1e-13)
    assert np.allclose(y.mean(axis=1), 0, atol=1e-13)
    assert np.allclose(y.var(axis=1), x.var(axis=1) / (x.var(axis=1) + eps), rtol=1e-12)
    # adding a constant to a row changes nothing; gamma and beta act as an affine map
    y2, _, _ = orc.layernorm_fwd(x + 3.5, np.ones(37), np.zeros(37), eps)
    assert np.allclose(y2, y, atol=1e-12)
    g, b = RNG.standard_normal(37), RNG.standard_normal(37)
    y3, _, _ = orc.layernorm_fwd(x, g, b, eps)
    assert np.allclose(y3, y * g + b, atol=1e-13)


@pytest.mark.parametrize("shape", [(1, 1), (3, 2), (6, 129)])
def test_layernorm_vs_pytorch_fp64(shape):
    import torch
    import torch.nn.functional as F
    rows, cols = shape
    x = torch.tensor(RNG.standard_normal(shape), requires_grad=True)
    g = torch.tensor(1 + 0.1 * RNG.standard_normal(cols), requires_grad=True)
    b = torch.tensor(0.1 * RNG.standard_normal(cols), requires_grad=True)
    dy = RNG.standard_normal(shape)
    y = F.layer_norm(x, (cols,), g, b, eps=1e-5)
    y.backward(torch.tensor(dy))
    yo, mean, rstd = orc.layernorm_fwd(x.detach().numpy(), g.detach().numpy(), b.detach().numpy(), 1e-5)
    assert np.allclose(yo, y.detach().numpy(), rtol=1e-11, atol=1e-12)
    dx, dg, db = orc.layernorm_bwd(x.detach().numpy(), dy, g.detach().numpy(), mean, rstd)
    assert np.allclose(dx, x.grad.numpy(), rtol=1e-9, atol=1e-10)
    assert np.allclose(dg, g.grad.numpy(), rtol=1e-10, atol=1e-11)
    assert np.allclose(db, b.grad.numpy(), rtol=1e-12, atol=1e-12)


def test_layernorm_backward_invariants():
    # dx of a row is orthogonal to the constant vector and (up to eps) to xhat
    x = RNG.standard_normal((4, 50))
    g = 1 + 0.1 * RNG.standard_normal(50)
    dy = RNG.standard_normal((4, 50))
    _, mean, rstd = orc.layernorm_fwd(x, g, np.zeros(50), 0.0)
    dx, _, _ = orc.layernorm_bwd(x, dy, g, mean, rstd)
    xh = (x - mean[:, None]) * rstd[:, None]
    assert np.allclose(dx.sum(axis=1), 0, atol=1e-12)
    assert np.allclose((dx * xh).sum(axis=1), 0, atol=1e-11)


# ------------------------------------------------------------------ softmax --

def test_softmax_invariants_and_closed_form():
    x = RNG.standard_normal((6, 41)) * 5
    y = orc.softmax_fwd(x)
    assert np.allclose(y.sum(axis=1), 1, atol=1e-14) and (y > 0).all()
    assert np.allclose(orc.softmax_fwd(x + 1000.0), y, atol=1e-13)  # shift invariance, no overflow
    # two entries: softmax([a, b])[0] = sigmoid(a - b)
    ab = np.array([[0.3, -1.1], [5.0, 5.0], [-700.0, 700.0]])
    y2 = orc.softmax_fwd(ab)
    with np.errstate(over="ignore"):
        assert np.allclose(y2[:, 0], 1 / (1 + np.exp(-(ab[:, 0] - ab[:, 1]))), atol=1e-15)
    # a single column is always 1
    assert np.array_equal(orc.softmax_fwd(np.array([[3.0], [-2.0]])), np.ones((2, 1)))


def test_softmax_vs_pytorch_fp64():
    import torch
    x = torch.tensor(RNG.standard_normal((9, 65)) * 3, requires_grad=True)
    dy = RNG.standard_normal((9, 65))
    y = torch.softmax(x, dim=-1)
    y.backward(torch.tensor(dy))
    yo = orc.softmax_fwd(x.detach().numpy())
    assert np.allclose(yo, y.detach().numpy(), rtol=1e-13, atol=1e-15)
    dx = orc.softmax_bwd(yo, dy)
    assert np.allclose(dx, x.grad.numpy(), rtol=1e-11, atol=1e-13)
    assert np.allclose(dx.sum(axis=1), 0, atol=1e-14)  # the Jacobian annihilates constants

"""Pins of the CPU oracle against things other than itself.

Each test checks the oracle against a closed form, an invariant, brute force on a
tiny input, finite differences, or a library routine.  Nothing here touches the
HIP path.
"""
import math

import numpy as np
import pytest

from mbconv_inputs import BlockShape, CONFIG0, make_block_inputs
from oracle import oracle as orc

RNG = np.random.default_rng(1234)


# ---------------------------------------------------------------- Swish ------

def test_swish_closed_forms():
    assert orc.swish(0.0) == 0.0
    assert orc.swish_grad(0.0) == 0.5
    for t in (0.1, 0.7, 1.3, 4.0, 11.0):
        # swish(t) - swish(-t) = t because sigmoid(t) + sigmoid(-t) = 1
        assert abs(orc.swish(t) - orc.swish(-t) - t) < 1e-14
        assert abs(orc.sigmoid(t) + orc.sigmoid(-t) - 1.0) < 1e-15
    assert abs(orc.swish(40.0) - 40.0) < 1e-12
    assert abs(orc.swish(-40.0)) < 1e-12
    assert abs(orc.swish(1.0) - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15


def test_swish_minimum():
    # the single stationary point solves 1 + t(1 - sigmoid(t)) = 0; bisection on swish_grad
    lo, hi = -2.0, -1.0
    assert orc.swish_grad(lo) < 0 < orc.swish_grad(hi)
    for _ in range(80):
        mid = 0.5 * (lo + hi)
        if orc.swish_grad(mid) < 0:
            lo = mid
        else:
            hi = mid
    t = 0.5 * (lo + hi)
    assert abs(t + 1.2784645) < 1e-6
    assert abs(orc.swish(t) + 0.2784645) < 1e-6
    s = 1.0 / (1.0 + math.exp(-t))
    assert abs(1.0 + t * (1.0 - s)) < 1e-12


def test_swish_grad_matches_finite_difference():
    for t in (-3.0, -1.2, -0.1, 0.4, 2.5):
        h = 1e-6
        fd = (orc.swish(t + h) - orc.swish(t - h)) / (2 * h)
        assert abs(fd - orc.swish_grad(t)) < 1e-9


# ------------------------------------------------------------- 1x1 conv ------

def test_conv1x1_is_a_matrix_product():
    x = RNG.standard_normal((3, 5, 4, 7))
    w = RNG.standard_normal((6, 5))
    ref = np.einsum("oi,nihw->nohw", w, x)
    assert np.allclose(orc.conv1x1(w, x), ref, rtol=0, atol=1e-13)
    dy = RNG.standard_normal((3, 6, 4, 7))
    assert np.allclose(orc.conv1x1_bwd_input(w, dy), np.einsum("oi,nohw->nihw", w, dy), atol=1e-13)
    assert np.allclose(orc.conv1x1_bwd_weight(x, dy), np.einsum("nohw,nihw->oi", dy, x),
                       atol=1e-12)


def test_conv1x1_not_transposed():
    # a weight matrix with a single 1 routes exactly one input channel to one output channel
    x = RNG.standard_normal((1, 3, 2, 2))
    w = np.zeros((2, 3))
    w[1, 2] = 1.0
    y = orc.conv1x1(w, x)
    assert np.array_equal(y[0, 1], x[0, 2]) and np.all(y[0, 0] == 0)


# ------------------------------------------------------------ depthwise ------

def _brute_depthwise(w, a, s, p):
    N, Cc, H, W = a.shape
    k = w.shape[-1]
    ap = np.zeros((N, Cc, H + 2 * p, W + 2 * p))
    ap[:, :, p:p + H, p:p + W] = a
    Ho, Wo = (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1
    d = np.zeros((N, Cc, Ho, Wo))
    for n in range(N):
        for c in range(Cc):
            for i in range(Ho):
                for j in range(Wo):
                    d[n, c, i, j] = np.sum(w[c] * ap[n, c, i * s:i * s + k, j * s:j * s + k])
    return d


@pytest.mark.parametrize("k,s,H,W", [(3, 1, 6, 5), (3, 2, 7, 6), (5, 1, 6, 7), (5, 2, 8, 7),
                                      (5, 2, 9, 9)])
def test_depthwise_vs_brute_force(k, s, H, W):
    p = (k - 1) // 2
    a = RNG.standard_normal((2, 3, H, W))
    w = RNG.standard_normal((3, k, k))
    assert np.allclose(orc.depthwise_fwd(w, a, s, p), _brute_depthwise(w, a, s, p), atol=1e-13)


@pytest.mark.parametrize("k", [3, 5])
def test_depthwise_delta_kernel(k):
    p = (k - 1) // 2
    a = RNG.standard_normal((1, 2, 8, 8))
    w = np.zeros((2, k, k))
    w[:, p, p] = 1.0
    assert np.array_equal(orc.depthwise_fwd(w, a, 1, p), a)
    assert np.array_equal(orc.depthwise_fwd(w, a, 2, p), a[:, :, ::2, ::2])
    # an off-centre delta shifts the image: out[i,j] = a[i+u-p, j+v-p]
    w2 = np.zeros((2, k, k))
    w2[:, 0, p + 1] = 1.0
    d = orc.depthwise_fwd(w2, a, 1, p)
    assert np.array_equal(d[:, :, p:, :-1], a[:, :, :8 - p, 1:])
    assert np.all(d[:, :, :p, :] == 0) and np.all(d[:, :, :, -1] == 0)


def test_depthwise_ones_counts_taps():
    a = np.ones((1, 1, 6, 6))
    d3 = orc.depthwise_fwd(np.ones((1, 3, 3)), a, 1, 1)[0, 0]
    assert d3[0, 0] == 4 and d3[0, 2] == 6 and d3[2, 2] == 9
    d5 = orc.depthwise_fwd(np.ones((1, 5, 5)), a, 1, 2)[0, 0]
    assert d5[0, 0] == 9 and d5[2, 2] == 25 and d5[0, 2] == 15 and d5[1, 1] == 16


@pytest.mark.parametrize("k,s", [(3, 1), (3, 2), (5, 1), (5, 2)])
def test_depthwise_backward_is_the_adjoint(k, s):
    # <dd, fwd(a)> = <bwd_input(dd), a> and = <bwd_weight(a, dd), w> (bilinear form)
    p = (k - 1) // 2
    H, W = 9, 8
    a = RNG.standard_normal((2, 3, H, W))
    w = RNG.standard_normal((3, k, k))
    d = orc.depthwise_fwd(w, a, s, p)
    dd = RNG.standard_normal(d.shape)
    lhs = np.sum(dd * d)
    assert abs(lhs - np.sum(orc.depthwise_bwd_input(w, dd, H, W, s, p) * a)) < 1e-11
    assert abs(lhs - np.sum(orc.depthwise_bwd_weight(a, dd, k, s, p) * w)) < 1e-11
    # brute-force gather form of the input gradient
    da = orc.depthwise_bwd_input(w, dd, H, W, s, p)
    ref = np.zeros_like(a)
    for h in range(H):
        for x in range(W):
            for u in range(k):
                for v in range(k):
                    ih, jw = h + p - u, x + p - v
                    if ih % s == 0 and jw % s == 0 and 0 <= ih // s < d.shape[2] \
                            and 0 <= jw // s < d.shape[3]:
                        ref[:, :, h, x] += w[:, u, v] * dd[:, :, ih // s, jw // s]
    assert np.allclose(da, ref, atol=1e-13)


# ------------------------------------------------------------ batch norm -----

def test_bn_invariants():
    x = 3.0 + 2.0 * RNG.standard_normal((4, 3, 5, 6))
    gamma, beta = RNG.standard_normal(3), RNG.standard_normal(3)
    eps = 1e-3
    y, xhat, mean, var, _, _ = orc.bn_fwd(x, gamma, beta, eps, 0.1)
    assert np.allclose(mean, x.mean(axis=(0, 2, 3)), atol=1e-13)
    assert np.allclose(var, x.var(axis=(0, 2, 3)), atol=1e-13)
    assert np.allclose(xhat.mean(axis=(0, 2, 3)), 0, atol=1e-13)
    assert np.allclose(xhat.var(axis=(0, 2, 3)), var / (var + eps), atol=1e-13)
    assert np.allclose(y, gamma[None, :, None, None] * xhat + beta[None, :, None, None])
    # eps = 0 gives variance exactly one
    _, xhat0, *_ = orc.bn_fwd(x, np.ones(3), np.zeros(3), 0.0, 0.1)
    assert np.allclose(xhat0.var(axis=(0, 2, 3)), 1.0, atol=1e-13)
    y1, xhat1, *_ = orc.bn_fwd(x, np.ones(3), np.zeros(3), eps, 0.1)
    assert np.array_equal(y1, xhat1)


def test_bn_running_statistics_closed_form():
    x = RNG.standard_normal((2, 2, 3, 3)) * 2 + 1
    rm0, rv0 = np.array([0.3, -0.2]), np.array([1.5, 0.7])
    alpha = 0.01
    m = 2 * 3 * 3
    *_, rm, rv = orc.bn_fwd(x, np.ones(2), np.zeros(2), 1e-3, alpha, rm0, rv0)
    assert np.allclose(rm, (1 - alpha) * rm0 + alpha * x.mean(axis=(0, 2, 3)), atol=1e-15)
    assert np.allclose(rv, (1 - alpha) * rv0 + alpha * x.var(axis=(0, 2, 3)) * m / (m - 1),
                       atol=1e-15)


def test_bn_backward_invariants_and_fd():
    x = RNG.standard_normal((3, 2, 4, 4)) + 0.5
    gamma, beta = np.array([1.3, 0.7]), np.array([0.1, -0.2])
    eps = 1e-3
    y, xhat, mean, var, _, _ = orc.bn_fwd(x, gamma, beta, eps, 0.1)
    dy = RNG.standard_normal(x.shape)
    dx, dgamma, dbeta = orc.bn_bwd(dy, xhat, gamma, var, eps)
    assert np.allclose(dbeta, dy.sum(axis=(0, 2, 3)))
    assert np.allclose(dgamma, (dy * xhat).sum(axis=(0, 2, 3)))
    assert np.allclose(dx.sum(axis=(0, 2, 3)), 0, atol=1e-12)
    # sum dx*xhat = gamma*rstd*dgamma*(1 - mean(xhat^2)) = gamma*rstd*dgamma*eps/(var+eps)
    assert np.allclose((dx * xhat).sum(axis=(0, 2, 3)),
                       gamma * dgamma * eps / (var + eps) ** 1.5, atol=1e-12)
    dx0 = orc.bn_bwd(dy, orc.bn_fwd(x, gamma, beta, 0.0, 0.1)[1], gamma, var, 0.0)[0]
    xh0 = orc.bn_fwd(x, gamma, beta, 0.0, 0.1)[1]
    assert np.allclose((dx0 * xh0).sum(axis=(0, 2, 3)), 0, atol=1e-12)
    # finite differences through the batch statistics
    h = 1e-6
    fd = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        xp, xm = x.copy(), x.copy()
        xp[i] += h
        xm[i] -= h
        fd[i] = (np.sum(orc.bn_fwd(xp, gamma, beta, eps, 0.1)[0] * dy)
                 - np.sum(orc.bn_fwd(xm, gamma, beta, eps, 0.1)[0] * dy)) / (2 * h)
    assert np.allclose(dx, fd, atol=1e-8)


# ------------------------------------------------------------------ SE -------

def test_se_on_spatially_constant_input():
    N, Cc, Cse = 2, 5, 3
    v = RNG.standard_normal((N, Cc))
    a2 = np.broadcast_to(v[:, :, None, None], (N, Cc, 4, 3)).copy()
    w1, b1 = RNG.standard_normal((Cse, Cc)), RNG.standard_normal(Cse)
    w2, b2 = RNG.standard_normal((Cc, Cse)), RNG.standard_normal(Cc)
    o = orc.se_fwd(a2, w1, b1, w2, b2)
    assert np.allclose(o.z, v, atol=1e-15)
    q = v @ w1.T + b1
    r = q / (1 + np.exp(-q))
    g = 1 / (1 + np.exp(-(r @ w2.T + b2)))
    assert np.allclose(o.g, g, atol=1e-14)
    assert np.allclose(o.sc, (v * g)[:, :, None, None] * np.ones((1, 1, 4, 3)), atol=1e-14)
    o0 = orc.se_fwd(a2, w1, b1, np.zeros_like(w2), np.zeros_like(b2))
    assert np.all(o0.g == 0.5)


def test_se_backward_fd():
    N, Cc, Cse = 2, 4, 2
    a2 = RNG.standard_normal((N, Cc, 3, 3))
    w1, b1 = RNG.standard_normal((Cse, Cc)), RNG.standard_normal(Cse)
    w2, b2 = RNG.standard_normal((Cc, Cse)), RNG.standard_normal(Cc)
    dsc = RNG.standard_normal(a2.shape)
    f = orc.se_fwd(a2, w1, b1, w2, b2)
    b = orc.se_bwd(a2, w1, w2, f, dsc)

    def loss(a2_, w1_, b1_, w2_, b2_):
        return np.sum(orc.se_fwd(a2_, w1_, b1_, w2_, b2_).sc * dsc)

    args = [a2, w1, b1, w2, b2]
    got = [b.da2, b.dw1, b.db1, b.dw2, b.db2]
    h = 1e-6
    for ai, g in enumerate(got):
        fd = np.zeros_like(args[ai])
        it = np.nditer(args[ai], flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            ap = [a.copy() for a in args]
            am = [a.copy() for a in args]
            ap[ai][i] += h
            am[ai][i] -= h
            fd[i] = (loss(*ap) - loss(*am)) / (2 * h)
        assert np.allclose(g, fd, atol=1e-8), ai


# --------------------------------------------------------- the whole block ---

def _tiny(**kw):
    base = dict(N=2, Cin=2, H=5, W=5, Cexp=4, Cse=2, Cout=2, k=3, stride=1, residual=True)
    base.update(kw)
    return BlockShape(**base)


TINY_SHAPES = [
    _tiny(),
    _tiny(k=5),
    _tiny(Cout=3, residual=False, stride=2),
    _tiny(Cout=3, residual=False, stride=2, k=5, H=6, W=7),
    _tiny(Cexp=2, has_expand=False),
    _tiny(Cexp=2, has_expand=False, residual=False, stride=2, Cout=3, k=5),
]


def _f64_inputs(s, seed=0):
    return {k: v.astype(np.float64) for k, v in make_block_inputs(s, seed).items()}


@pytest.mark.parametrize("s", TINY_SHAPES, ids=lambda s: f"k{s.k}s{s.stride}e{int(s.has_expand)}")
def test_block_gradients_vs_finite_differences(s):
    t = _f64_inputs(s, seed=3)
    f, b = orc.mbconv_step(s, t)
    dout = t["dout"]

    def loss(tt):
        return float(np.sum(orc.mbconv_forward(s, tt).out * dout))

    h = 1e-5
    names = ["x"] + [n for n in b.grads]
    for name in names:
        got = b.dx if name == "x" else b.grads[name]
        fd = np.zeros_like(t[name])
        it = np.nditer(t[name], flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            tp, tm = dict(t), dict(t)
            tp[name] = t[name].copy()
            tm[name] = t[name].copy()
            tp[name][i] += h
            tm[name][i] -= h
            fd[i] = (loss(tp) - loss(tm)) / (2 * h)
        scale = max(np.abs(fd).max(), 1e-3)
        assert np.abs(got - fd).max() / scale < 2e-6, (name, np.abs(got - fd).max(), scale)


def test_block_residual_with_gamma3_zero():
    s = _tiny()
    t = _f64_inputs(s)
    t["bn3_gamma"] = np.zeros_like(t["bn3_gamma"])
    f, b = orc.mbconv_step(s, t)
    assert np.allclose(f.out, t["bn3_beta"][None, :, None, None] + t["x"], atol=1e-15)
    # with gamma3 = 0 nothing flows through the main branch: dX is exactly dOut
    assert np.allclose(b.dx, t["dout"], atol=1e-15)
    assert np.allclose(b.grads["bn3_beta"], t["dout"].sum(axis=(0, 2, 3)))


def test_block_backward_linear_in_dout():
    s = _tiny(k=5)
    t = _f64_inputs(s)
    f = orc.mbconv_forward(s, t)
    d1 = RNG.standard_normal(t["dout"].shape)
    d2 = RNG.standard_normal(t["dout"].shape)
    b1 = orc.mbconv_backward(s, t, f.tape, d1)
    b2 = orc.mbconv_backward(s, t, f.tape, d2)
    b3 = orc.mbconv_backward(s, t, f.tape, 2.0 * d1 - 0.5 * d2)
    assert np.allclose(b3.dx, 2.0 * b1.dx - 0.5 * b2.dx, atol=1e-12)
    for n in b1.grads:
        assert np.allclose(b3.grads[n], 2.0 * b1.grads[n] - 0.5 * b2.grads[n], atol=1e-11)
    assert np.allclose(b1.grads["bn3_beta"], d1.sum(axis=(0, 2, 3)))


def test_block_bn_invariants_inside_the_block():
    s = CONFIG0
    t = make_block_inputs(s, 0)
    f = orc.mbconv_forward(s, t)
    for i, name in ((1, "xhat1"), (2, "xhat2"), (3, "xhat3")):
        xh = f.tape[name]
        var = f.tape[f"var{i}"]
        assert np.allclose(xh.mean(axis=(0, 2, 3)), 0, atol=1e-12)
        assert np.allclose(xh.var(axis=(0, 2, 3)), var / (var + s.eps), atol=1e-12)
    # running statistics started at (0, 1)
    m = s.N * s.Ho * s.Wo
    assert np.allclose(f.running["bn3_mean"], s.momentum * f.tape["mean3"])
    assert np.allclose(f.running["bn3_var"],
                       (1 - s.momentum) + s.momentum * f.tape["var3"] * m / (m - 1))


_MBV2 = [BlockShape(N=2, Cin=8, H=10, W=12, Cexp=48, Cse=1, Cout=8, k=3, stride=1, residual=True,
                    activation="relu6", has_se=False),
         BlockShape(N=3, Cin=8, H=9, W=9, Cexp=24, Cse=1, Cout=12, k=3, stride=2, residual=False,
                    activation="relu6", has_se=False),
         BlockShape(N=2, Cin=16, H=8, W=8, Cexp=16, Cse=1, Cout=8, k=3, stride=1, has_expand=False,
                    residual=False, activation="relu6", has_se=False),
         # the two switches are independent: ReLU6 with the SE stage, Swish without it
         BlockShape(N=2, Cin=8, H=7, W=7, Cexp=24, Cse=2, Cout=8, k=5, stride=1, residual=True,
                    activation="relu6"),
         BlockShape(N=2, Cin=8, H=7, W=7, Cexp=24, Cse=1, Cout=8, k=3, stride=1, residual=True,
                    has_se=False)]
_MBV2_IDS = ["mbv2_s1", "mbv2_s2", "mbv2_t1", "relu6_se", "swish_nose"]


def _torch_block(s, t):
    """The same block assembled from PyTorch CPU float64 library ops with autograd."""
    import torch
    import torch.nn.functional as F

    tt = {k: torch.tensor(np.asarray(v, dtype=np.float64), requires_grad=(k in orc._PARAMS
                                                                          or k == "x"))
          for k, v in t.items()}
    x = tt["x"]
    run = {n: tt[n].detach().clone() for n in orc._RUNNING}

    def bn(v, i):
        return F.batch_norm(v, run[f"bn{i}_mean"], run[f"bn{i}_var"], tt[f"bn{i}_gamma"],
                            tt[f"bn{i}_beta"], training=True, momentum=s.momentum, eps=s.eps)

    act = F.relu6 if s.activation == "relu6" else F.silu
    a = x
    if s.has_expand:
        a = act(bn(F.conv2d(a, tt["w_expand"][:, :, None, None]), 1))
    a = F.conv2d(a, tt["w_dw"][:, None], stride=s.stride, padding=s.pad, groups=s.Cexp)
    a = act(bn(a, 2))
    if s.has_se:
        z = a.mean(dim=(2, 3))
        r = F.silu(z @ tt["se_w1"].T + tt["se_b1"])
        g = torch.sigmoid(r @ tt["se_w2"].T + tt["se_b2"])
        a = a * g[:, :, None, None]
    out = bn(F.conv2d(a, tt["w_proj"][:, :, None, None]), 3)
    if s.residual:
        out = out + x
    (out * tt["dout"]).sum().backward()
    grads = {n: tt[n].grad.numpy() for n in orc._PARAMS if n in tt}
    return out.detach().numpy(), tt["x"].grad.numpy(), grads, {n: v.numpy() for n, v in run.items()}


@pytest.mark.parametrize("s", [CONFIG0, _tiny(Cout=3, residual=False, stride=2, k=5, H=8, W=8),
                               BlockShape(N=3, Cin=8, H=9, W=9, Cexp=8, Cse=2, Cout=8, k=3,
                                          stride=1, has_expand=False, residual=True)] + _MBV2,
                         ids=["config0", "k5s2", "noexpand"] + _MBV2_IDS)
def test_block_vs_pytorch_fp64_autograd(s):
    t = make_block_inputs(s, 0)
    f, b = orc.mbconv_step(s, t)
    out, dx, grads, run = _torch_block(s, t)
    assert np.allclose(f.out, out, rtol=1e-10, atol=1e-11)
    assert np.allclose(b.dx, dx, rtol=1e-9, atol=1e-10)
    for n, g in grads.items():
        assert np.allclose(b.grads[n], g, rtol=1e-9, atol=1e-9), n
    for n in orc._RUNNING:
        if s.has_expand or not n.startswith("bn1"):
            assert np.allclose(f.running[n], run[n], rtol=1e-12, atol=1e-13), n


# ------------------------------------------------------ evaluation mode ------

def _random_running(s, seed):
    """Running statistics that are neither (0, 1) nor the batch's own."""
    rng = np.random.default_rng(seed)
    run = {}
    for i, C_ in ((1, s.Cexp), (2, s.Cexp), (3, s.Cout)):
        run[f"bn{i}_mean"] = 0.3 * rng.standard_normal(C_)
        run[f"bn{i}_var"] = 0.5 + rng.random(C_)
    return run


def test_bn_eval_closed_form():
    # one value per channel: (x - m)/sqrt(v + eps) written out by hand
    x = np.array([[[[2.0]], [[-1.0]]]])
    y = orc.bn_eval(x, np.array([3.0, 0.5]), np.array([0.25, -2.0]), 0.21,
                    np.array([0.5, 1.0]), np.array([0.04, 1.0]))
    assert abs(y[0, 0, 0, 0] - (3.0 * (2.0 - 0.5) / 0.5 + 0.25)) < 1e-14
    assert abs(y[0, 1, 0, 0] - (0.5 * (-1.0 - 1.0) / 1.1 - 2.0)) < 1e-14
    # running statistics (0, 1 - eps) make it the affine map gamma*x + beta
    x = RNG.standard_normal((2, 3, 4, 5))
    g, b = RNG.standard_normal(3), RNG.standard_normal(3)
    y = orc.bn_eval(x, g, b, 1e-3, np.zeros(3), np.full(3, 1.0 - 1e-3))
    assert np.allclose(y, g[None, :, None, None] * x + b[None, :, None, None], atol=1e-13)


@pytest.mark.parametrize("s", [CONFIG0, _tiny(Cout=3, residual=False, stride=2, k=5, H=8, W=8),
                               BlockShape(N=3, Cin=8, H=9, W=9, Cexp=8, Cse=2, Cout=8, k=3,
                                          stride=1, has_expand=False, residual=True)] + _MBV2,
                         ids=["config0", "k5s2", "noexpand"] + _MBV2_IDS)
def test_eval_block_with_batch_statistics_is_the_training_block(s):
    # Training mode normalises with the batch mean and the biased batch variance; handing
    # exactly those to the evaluation-mode block must reproduce the training output.
    t = make_block_inputs(s, 3)
    f = orc.mbconv_forward(s, t)
    run = {}
    for i in (1, 2, 3):
        if i == 1 and not s.has_expand:
            continue
        run[f"bn{i}_mean"] = f.tape[f"mean{i}"]
        run[f"bn{i}_var"] = f.tape[f"var{i}"]
    out = orc.mbconv_forward_eval(s, t, run)
    assert np.allclose(out, f.out, rtol=1e-11, atol=1e-12)
    # and different statistics must change it (the argument is really used)
    other = orc.mbconv_forward_eval(s, t, _random_running(s, 5))
    assert np.abs(other - f.out).max() > 1e-3


@pytest.mark.parametrize("s", [CONFIG0, _tiny(Cout=3, residual=False, stride=2, k=5, H=8, W=8),
                               BlockShape(N=3, Cin=8, H=9, W=9, Cexp=8, Cse=2, Cout=8, k=3,
                                          stride=1, has_expand=False, residual=True)] + _MBV2,
                         ids=["config0", "k5s2", "noexpand"] + _MBV2_IDS)
def test_eval_block_vs_pytorch_fp64(s):
    import torch
    import torch.nn.functional as F

    t = make_block_inputs(s, 0)
    run = _random_running(s, 11)
    tt = {k: torch.tensor(np.asarray(v, dtype=np.float64)) for k, v in {**t, **run}.items()}

    def bn(v, i):
        return F.batch_norm(v, tt[f"bn{i}_mean"], tt[f"bn{i}_var"], tt[f"bn{i}_gamma"],
                            tt[f"bn{i}_beta"], training=False, eps=s.eps)

    x = tt["x"]
    act = F.relu6 if s.activation == "relu6" else F.silu
    a = x
    if s.has_expand:
        a = act(bn(F.conv2d(a, tt["w_expand"][:, :, None, None]), 1))
    a = F.conv2d(a, tt["w_dw"][:, None], stride=s.stride, padding=s.pad, groups=s.Cexp)
    a = act(bn(a, 2))
    if s.has_se:
        z = a.mean(dim=(2, 3))
        r = F.silu(z @ tt["se_w1"].T + tt["se_b1"])
        g = torch.sigmoid(r @ tt["se_w2"].T + tt["se_b2"])
        a = a * g[:, :, None, None]
    out = bn(F.conv2d(a, tt["w_proj"][:, :, None, None]), 3)
    if s.residual:
        out = out + x
    got = orc.mbconv_forward_eval(s, t, run)
    assert np.allclose(got, out.numpy(), rtol=1e-10, atol=1e-11)


# ------------------------------------------- ReLU6, no squeeze-and-excitation ------

def test_relu6_closed_forms():
    for t, v, g in ((-2.0, 0.0, 0.0), (-1e-9, 0.0, 0.0), (0.0, 0.0, 0.0), (1e-9, 1e-9, 1.0),
                    (3.25, 3.25, 1.0), (6.0 - 1e-9, 6.0 - 1e-9, 1.0), (6.0, 6.0, 0.0),
                    (7.5, 6.0, 0.0)):
        assert orc.relu6(t) == v
        assert orc.relu6_grad(t) == g


def test_block_without_se_is_the_se_block_with_gate_one():
    # W2 = 0 and b2 = 40 make the gate sigmoid(40) = 1 - 4e-18: the block with the SE stage
    # then computes what the block without it computes, and the remaining gradients agree.
    s = _tiny()
    t = make_block_inputs(s, 9)
    t["se_w2"] = np.zeros_like(t["se_w2"])
    t["se_b2"] = np.full_like(t["se_b2"], 40.0)
    f1, b1 = orc.mbconv_step(s, t)
    from dataclasses import replace
    s0 = replace(s, has_se=False)
    t0 = {k: v for k, v in t.items() if not k.startswith("se_")}
    f0, b0 = orc.mbconv_step(s0, t0)
    assert np.allclose(f0.out, f1.out, rtol=1e-13, atol=1e-13)
    assert np.allclose(b0.dx, b1.dx, rtol=1e-12, atol=1e-13)
    for n, g in b0.grads.items():
        assert np.allclose(g, b1.grads[n], rtol=1e-12, atol=1e-12), n


def test_relu6_block_inside_the_linear_range_is_the_linear_block():
    # Betas of 3 and small gammas keep every pre-activation inside (0, 6), where ReLU6 is the
    # identity: the block is then conv -> BN -> depthwise -> BN -> conv -> BN assembled from
    # the separately pinned primitives.
    s = BlockShape(N=2, Cin=6, H=7, W=7, Cexp=12, Cse=1, Cout=6, k=3, stride=1, residual=True,
                   activation="relu6", has_se=False)
    t = make_block_inputs(s, 4)
    for i in (1, 2):
        t[f"bn{i}_gamma"] = (0.2 * t[f"bn{i}_gamma"]).astype(np.float32)
        t[f"bn{i}_beta"] = np.full_like(t[f"bn{i}_beta"], 3.0)
    f = orc.mbconv_forward(s, t)
    assert f.tape["y1"].min() > 0 and f.tape["y1"].max() < 6
    assert f.tape["y2"].min() > 0 and f.tape["y2"].max() < 6
    e = orc.conv1x1(t["w_expand"], t["x"])
    y1 = orc.bn_fwd(e, t["bn1_gamma"], t["bn1_beta"], s.eps, s.momentum)[0]
    d = orc.depthwise_fwd(t["w_dw"], y1, s.stride, s.pad)
    y2 = orc.bn_fwd(d, t["bn2_gamma"], t["bn2_beta"], s.eps, s.momentum)[0]
    p = orc.conv1x1(t["w_proj"], y2)
    out = orc.bn_fwd(p, t["bn3_gamma"], t["bn3_beta"], s.eps, s.momentum)[0] + t["x"]
    assert np.allclose(f.out, out, rtol=1e-12, atol=1e-12)

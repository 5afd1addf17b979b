"""ctypes front end of the fp64 CPU oracle (``mbconv_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Only the tests, ``__graft_entry__.smoke`` and the
``cpu_baseline`` leg of ``bench.py`` may import this module; the product package
never does, and this module imports nothing from the product package.

Every function takes and returns numpy float64 arrays (NCHW, contiguous).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from types import SimpleNamespace

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mbconv_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_mbconv.so")

_dp = C.POINTER(C.c_double)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C99 + OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall",
                               "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Desc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("N", "Cin", "H", "W", "Cexp", "Cse", "Cout", "k", "stride",
                                        "pad", "has_expand", "residual")] + \
               [("eps", C.c_double), ("momentum", C.c_double), ("activation", C.c_int),
                ("has_se", C.c_int)]


_PARAMS = ["w_expand", "bn1_gamma", "bn1_beta", "w_dw", "bn2_gamma", "bn2_beta", "se_w1", "se_b1",
           "se_w2", "se_b2", "w_proj", "bn3_gamma", "bn3_beta"]
_RUNNING = ["bn1_mean", "bn1_var", "bn2_mean", "bn2_var", "bn3_mean", "bn3_var"]
_TAPE = ["e", "xhat1", "y1", "a1", "d", "xhat2", "y2", "a2", "sc", "z", "t", "g", "q", "r", "p",
         "xhat3", "mean1", "var1", "mean2", "var2", "mean3", "var3"]


class _Params(C.Structure):
    _fields_ = [(n, _dp) for n in _PARAMS]


class _Grads(C.Structure):
    _fields_ = [(n, _dp) for n in _PARAMS]


class _Running(C.Structure):
    _fields_ = [(n, _dp) for n in _RUNNING]


class _Tape(C.Structure):
    _fields_ = [(n, _dp) for n in _TAPE]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        for name in ("orc_sigmoid", "orc_swish", "orc_swish_grad", "orc_relu6", "orc_relu6_grad"):
            f = getattr(_lib, name)
            f.restype = C.c_double
            f.argtypes = [C.c_double]
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: np.ndarray):
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_dp)


def num_threads() -> int:
    return int(lib().orc_num_threads())


# ---- scalar functions ---------------------------------------------------------

def relu6(t: float) -> float:
    return float(lib().orc_relu6(float(t)))


def relu6_grad(t: float) -> float:
    return float(lib().orc_relu6_grad(float(t)))


def sigmoid(t: float) -> float:
    return lib().orc_sigmoid(float(t))


def swish(t: float) -> float:
    return lib().orc_swish(float(t))


def swish_grad(t: float) -> float:
    return lib().orc_swish_grad(float(t))


# ---- single steps (used by the pins) ------------------------------------------

def conv1x1(w, x):
    w, x = _f64(w), _f64(x)
    N, Ci, H, W = x.shape
    Co = w.shape[0]
    y = np.empty((N, Co, H, W))
    lib().orc_conv1x1(N, Ci, Co, H * W, _p(w), _p(x), _p(y))
    return y


def conv1x1_bwd_input(w, dy):
    w, dy = _f64(w), _f64(dy)
    N, Co, H, W = dy.shape
    Ci = w.shape[1]
    dx = np.empty((N, Ci, H, W))
    lib().orc_conv1x1_bwd_input(N, Ci, Co, H * W, _p(w), _p(dy), _p(dx))
    return dx


def conv1x1_bwd_weight(x, dy):
    x, dy = _f64(x), _f64(dy)
    N, Ci, H, W = x.shape
    Co = dy.shape[1]
    dw = np.empty((Co, Ci))
    lib().orc_conv1x1_bwd_weight(N, Ci, Co, H * W, _p(x), _p(dy), _p(dw))
    return dw


def bn_fwd(x, gamma, beta, eps, momentum, run_mean=None, run_var=None):
    """Returns (y, xhat, mean, var_biased, new_run_mean, new_run_var)."""
    x, gamma, beta = _f64(x), _f64(gamma), _f64(beta)
    N, Cc, H, W = x.shape
    mean, var = np.empty(Cc), np.empty(Cc)
    xhat, y = np.empty_like(x), np.empty_like(x)
    rm = _f64(run_mean).copy() if run_mean is not None else None
    rv = _f64(run_var).copy() if run_var is not None else None
    lib().orc_bn_fwd(N, Cc, H * W, _p(x), _p(gamma), _p(beta), C.c_double(eps),
                     C.c_double(momentum), _p(mean), _p(var), _p(rm) if rm is not None else None,
                     _p(rv) if rv is not None else None, _p(xhat), _p(y))
    return y, xhat, mean, var, rm, rv


def bn_bwd(dy, xhat, gamma, var, eps):
    dy, xhat, gamma, var = _f64(dy), _f64(xhat), _f64(gamma), _f64(var)
    N, Cc, H, W = dy.shape
    dx, dgamma, dbeta = np.empty_like(dy), np.empty(Cc), np.empty(Cc)
    lib().orc_bn_bwd(N, Cc, H * W, _p(dy), _p(xhat), _p(gamma), _p(var), C.c_double(eps), _p(dx),
                     _p(dgamma), _p(dbeta))
    return dx, dgamma, dbeta


def _out_hw(H, W, k, s, p):
    return (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1


def depthwise_fwd(w, a, stride, pad):
    w, a = _f64(w), _f64(a)
    N, Cc, H, W = a.shape
    k = w.shape[-1]
    Ho, Wo = _out_hw(H, W, k, stride, pad)
    d = np.empty((N, Cc, Ho, Wo))
    lib().orc_depthwise_fwd(N, Cc, H, W, k, stride, pad, _p(w), _p(a), _p(d))
    return d


def depthwise_bwd_input(w, dd, H, W, stride, pad):
    w, dd = _f64(w), _f64(dd)
    N, Cc = dd.shape[:2]
    k = w.shape[-1]
    da = np.empty((N, Cc, H, W))
    lib().orc_depthwise_bwd_input(N, Cc, H, W, k, stride, pad, _p(w), _p(dd), _p(da))
    return da


def depthwise_bwd_weight(a, dd, k, stride, pad):
    a, dd = _f64(a), _f64(dd)
    N, Cc, H, W = a.shape
    dw = np.empty((Cc, k, k))
    lib().orc_depthwise_bwd_weight(N, Cc, H, W, k, stride, pad, _p(a), _p(dd), _p(dw))
    return dw


def se_fwd(a2, w1, b1, w2, b2):
    """Returns a namespace with z, q, r, t, g, sc."""
    a2, w1, b1, w2, b2 = map(_f64, (a2, w1, b1, w2, b2))
    N, Cc, H, W = a2.shape
    Cse = w1.shape[0]
    o = SimpleNamespace(z=np.empty((N, Cc)), q=np.empty((N, Cse)), r=np.empty((N, Cse)),
                        t=np.empty((N, Cc)), g=np.empty((N, Cc)), sc=np.empty_like(a2))
    lib().orc_se_fwd(N, Cc, Cse, H * W, _p(a2), _p(w1), _p(b1), _p(w2), _p(b2), _p(o.z), _p(o.q),
                     _p(o.r), _p(o.t), _p(o.g), _p(o.sc))
    return o


def se_bwd(a2, w1, w2, fwd, dsc):
    a2, w1, w2, dsc = map(_f64, (a2, w1, w2, dsc))
    N, Cc, H, W = a2.shape
    Cse = w1.shape[0]
    o = SimpleNamespace(da2=np.empty_like(a2), dw1=np.empty((Cse, Cc)), db1=np.empty(Cse),
                        dw2=np.empty((Cc, Cse)), db2=np.empty(Cc))
    lib().orc_se_bwd(N, Cc, Cse, H * W, _p(a2), _p(w1), _p(w2), _p(fwd.z), _p(fwd.q), _p(fwd.r),
                     _p(fwd.g), _p(dsc), _p(o.da2), _p(o.dw1), _p(o.db1), _p(o.dw2), _p(o.db2))
    return o


# ---- the whole block ------------------------------------------------------------

def _desc(s) -> _Desc:
    return _Desc(s.N, s.Cin, s.H, s.W, s.Cexp, s.Cse, s.Cout, s.k, s.stride, s.pad,
                 int(s.has_expand), int(s.residual), float(s.eps), float(s.momentum),
                 1 if getattr(s, "activation", "swish") == "relu6" else 0,
                 int(getattr(s, "has_se", True)))


def _params_struct(s, t, keep):
    ps = _Params()
    for n in _PARAMS:
        if n in t:
            a = _f64(t[n])
            keep.append(a)
            setattr(ps, n, _p(a))
    return ps


def mbconv_forward(s, t):
    """One training-mode forward.  ``s`` is a BlockShape-like object, ``t`` a dict with x, the
    parameters and (optionally) the six running statistics.

    Returns a namespace: out, tape (dict of every intermediate), running (dict, updated copies).
    """
    keep = []
    x = _f64(t["x"])
    ps = _params_struct(s, t, keep)
    E = (s.N, s.Cexp, s.H, s.W)
    D = (s.N, s.Cexp, s.Ho, s.Wo)
    P = (s.N, s.Cout, s.Ho, s.Wo)
    shapes = dict(e=E, xhat1=E, y1=E, a1=E, d=D, xhat2=D, y2=D, a2=D, sc=D, z=(s.N, s.Cexp),
                  t=(s.N, s.Cexp), g=(s.N, s.Cexp), q=(s.N, s.Cse), r=(s.N, s.Cse), p=P, xhat3=P,
                  mean1=(s.Cexp,), var1=(s.Cexp,), mean2=(s.Cexp,), var2=(s.Cexp,),
                  mean3=(s.Cout,), var3=(s.Cout,))
    if not s.has_expand:
        for n in ("e", "xhat1", "y1", "mean1", "var1"):
            shapes[n] = (1,)
    tape = {n: np.zeros(sh) for n, sh in shapes.items()}
    ts = _Tape()
    for n in _TAPE:
        setattr(ts, n, _p(tape[n]))
    running = {}
    rs = _Running()
    for n in _RUNNING:
        C_ = s.Cout if n.startswith("bn3") else s.Cexp
        default = np.ones(C_) if n.endswith("var") else np.zeros(C_)
        running[n] = _f64(t[n]).copy() if n in t else default
        setattr(rs, n, _p(running[n]))
    out = np.empty(P)
    d = _desc(s)
    rc = lib().orc_mbconv_forward(C.byref(d), C.byref(ps), C.byref(rs), _p(x), _p(out),
                                  C.byref(ts))
    if rc != 0:
        raise ValueError(f"orc_mbconv_forward returned {rc}")
    return SimpleNamespace(out=out, tape=tape, running=running)


def bn_eval(x, gamma, beta, eps, run_mean, run_var):
    """Evaluation-mode BN: gamma*(x-run_mean)/sqrt(run_var+eps)+beta."""
    x = _f64(x)
    N, Cc, H, W = x.shape
    y = np.empty_like(x)
    lib().orc_bn_eval(N, Cc, H * W, _p(x), _p(_f64(gamma)), _p(_f64(beta)), C.c_double(eps),
                      _p(_f64(run_mean)), _p(_f64(run_var)), _p(y))
    return y


def mbconv_forward_eval(s, t, running=None):
    """Evaluation-mode forward: every BN uses the running statistics (``running`` dict, else the
    entries of ``t``, else mean 0 / variance 1).  Returns out."""
    keep = []
    x = _f64(t["x"])
    ps = _params_struct(s, t, keep)
    rs = _Running()
    for n in _RUNNING:
        C_ = s.Cout if n.startswith("bn3") else s.Cexp
        default = np.ones(C_) if n.endswith("var") else np.zeros(C_)
        src = running if (running is not None and n in running) else t
        a = _f64(src[n]).copy() if n in src else default
        keep.append(a)
        setattr(rs, n, _p(a))
    out = np.empty((s.N, s.Cout, s.Ho, s.Wo))
    d = _desc(s)
    rc = lib().orc_mbconv_forward_eval(C.byref(d), C.byref(ps), C.byref(rs), _p(x), _p(out))
    if rc != 0:
        raise ValueError(f"orc_mbconv_forward_eval returned {rc}")
    return out


def mbconv_backward(s, t, tape, dout=None):
    """Backward of ``mbconv_forward``.  Returns a namespace: dx, grads (dict)."""
    keep = []
    x = _f64(t["x"])
    dout = _f64(t["dout"] if dout is None else dout)
    ps = _params_struct(s, t, keep)
    ts = _Tape()
    for n in _TAPE:
        setattr(ts, n, _p(tape[n]))
    grads = {}
    gs = _Grads()
    for n in _PARAMS:
        if n in t:
            grads[n] = np.zeros(np.shape(t[n]))
            setattr(gs, n, _p(grads[n]))
    dx = np.empty(x.shape)
    d = _desc(s)
    rc = lib().orc_mbconv_backward(C.byref(d), C.byref(ps), _p(x), _p(dout), C.byref(ts), _p(dx),
                                   C.byref(gs))
    if rc != 0:
        raise ValueError(f"orc_mbconv_backward returned {rc}")
    return SimpleNamespace(dx=dx, grads=grads)


def mbconv_step(s, t):
    """Forward + backward; returns (forward namespace, backward namespace)."""
    f = mbconv_forward(s, t)
    b = mbconv_backward(s, t, f.tape)
    return f, b

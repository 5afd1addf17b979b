"""ctypes front end of the fp64 CPU oracle for Mish, layer normalisation and softmax
(``dnnops_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Only the tests, ``__graft_entry__.smoke`` and the ``cpu_baseline``
leg of ``bench.py`` may import this module; the product package never does, and this module
imports nothing from the product package.  numpy float64 arrays in and out.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dnnops_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_dnnops.so")
_dp = C.POINTER(C.c_double)
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall",
                               "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        for name in ("orc_mish", "orc_mish_grad"):
            f = getattr(_lib, name)
            f.restype = C.c_double
            f.argtypes = [C.c_double]
    return _lib


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_dp)


def mish(x: float) -> float:
    return float(lib().orc_mish(float(x)))


def mish_grad(x: float) -> float:
    return float(lib().orc_mish_grad(float(x)))


def mish_fwd(x):
    x = _f64(x)
    y = np.empty_like(x)
    lib().orc_mish_fwd(C.c_size_t(x.size), _p(x), _p(y))
    return y


def mish_bwd(x, dy):
    x, dy = _f64(x), _f64(dy)
    dx = np.empty_like(x)
    lib().orc_mish_bwd(C.c_size_t(x.size), _p(x), _p(dy), _p(dx))
    return dx


def layernorm_fwd(x, gamma, beta, eps):
    """x [rows, cols]; returns (y, mean[rows], rstd[rows])."""
    x, gamma, beta = _f64(x), _f64(gamma), _f64(beta)
    rows, cols = x.shape
    y, mean, rstd = np.empty_like(x), np.empty(rows), np.empty(rows)
    lib().orc_layernorm_fwd(rows, cols, _p(x), _p(gamma), _p(beta), C.c_double(eps), _p(y),
                            _p(mean), _p(rstd))
    return y, mean, rstd


def layernorm_bwd(x, dy, gamma, mean, rstd):
    """Returns (dx, dgamma, dbeta)."""
    x, dy, gamma, mean, rstd = _f64(x), _f64(dy), _f64(gamma), _f64(mean), _f64(rstd)
    rows, cols = x.shape
    dx, dgamma, dbeta = np.empty_like(x), np.empty(cols), np.empty(cols)
    lib().orc_layernorm_bwd(rows, cols, _p(x), _p(dy), _p(gamma), _p(mean), _p(rstd), _p(dx),
                            _p(dgamma), _p(dbeta))
    return dx, dgamma, dbeta


def softmax_fwd(x):
    x = _f64(x)
    rows, cols = x.shape
    y = np.empty_like(x)
    lib().orc_softmax_fwd(rows, cols, _p(x), _p(y))
    return y


def softmax_bwd(y, dy):
    y, dy = _f64(y), _f64(dy)
    rows, cols = y.shape
    dx = np.empty_like(y)
    lib().orc_softmax_bwd(rows, cols, _p(y), _p(dy), _p(dx))
    return dx

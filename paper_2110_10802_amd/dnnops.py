"""ctypes binding of the Mish / layer-normalisation / softmax entry points of libmbconv.so
(argument marshalling only; mirrors include/dnnops.h one to one).  Tensors are anything with a
``data_ptr()`` method.  There is no fallback: if the HIP library is missing, loading raises."""
from __future__ import annotations

import ctypes as C
from typing import Any

from . import binding as _B

EXPORTS = ["dnnops_mish_forward", "dnnops_mish_backward", "dnnops_layernorm_forward",
           "dnnops_layernorm_backward_scratch_bytes", "dnnops_layernorm_backward",
           "dnnops_layernorm_backward_noalloc_max_scratch_bytes", "dnnops_layernorm_backward_noalloc",
           "dnnops_softmax_forward", "dnnops_softmax_backward"]
MAX_COLS = 8192
_ready = False


class DnnOpsError(RuntimeError):
    def __init__(self, status: int, where: str):
        super().__init__(f"{where}: status {status}")
        self.status = status


def load():
    global _ready
    lib = _B.load()
    if not _ready:
        vp, f, i32 = C.c_void_p, C.c_float, C.c_int32
        lib.dnnops_mish_forward.argtypes = [vp, vp, C.c_size_t, vp]
        lib.dnnops_mish_backward.argtypes = [vp, vp, vp, C.c_size_t, vp]
        lib.dnnops_layernorm_forward.argtypes = [vp, vp, vp, f, i32, i32, vp, vp, vp, vp]
        lib.dnnops_layernorm_backward_scratch_bytes.argtypes = [i32, i32]
        lib.dnnops_layernorm_backward_scratch_bytes.restype = C.c_size_t
        lib.dnnops_layernorm_backward.argtypes = [vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp]
        lib.dnnops_layernorm_backward_noalloc.argtypes = [vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp]
        lib.dnnops_layernorm_backward_noalloc_max_scratch_bytes.argtypes = []
        lib.dnnops_layernorm_backward_noalloc_max_scratch_bytes.restype = C.c_size_t
        lib.dnnops_softmax_forward.argtypes = [vp, vp, i32, i32, vp]
        lib.dnnops_softmax_backward.argtypes = [vp, vp, vp, i32, i32, vp]
        for n in EXPORTS:
            if not n.endswith("scratch_bytes"):
                getattr(lib, n).restype = C.c_int
        _ready = True
    return lib


def _ptr(t: Any):
    if t is None or isinstance(t, int):
        return t
    return int(t.data_ptr())


def _check(rc: int, where: str):
    if rc != 0:
        raise DnnOpsError(rc, where)


def mish_forward(x, y, n: int, stream: int = 0) -> None:
    _check(load().dnnops_mish_forward(_ptr(x), _ptr(y), n, stream or None), "dnnops_mish_forward")


def mish_backward(x, dy, dx, n: int, stream: int = 0) -> None:
    _check(load().dnnops_mish_backward(_ptr(x), _ptr(dy), _ptr(dx), n, stream or None),
           "dnnops_mish_backward")


def layernorm_forward(x, gamma, beta, eps: float, rows: int, cols: int, y, mean, rstd,
                      stream: int = 0) -> None:
    _check(load().dnnops_layernorm_forward(_ptr(x), _ptr(gamma), _ptr(beta), eps, rows, cols, _ptr(y),
                                           _ptr(mean), _ptr(rstd), stream or None),
           "dnnops_layernorm_forward")


def layernorm_backward_scratch_bytes(rows: int, cols: int) -> int:
    return int(load().dnnops_layernorm_backward_scratch_bytes(rows, cols))


def layernorm_backward(x, dy, gamma, mean, rstd, rows: int, cols: int, dx, dgamma, dbeta, scratch,
                       stream: int = 0) -> None:
    _check(load().dnnops_layernorm_backward(_ptr(x), _ptr(dy), _ptr(gamma), _ptr(mean), _ptr(rstd),
                                            rows, cols, _ptr(dx), _ptr(dgamma), _ptr(dbeta),
                                            _ptr(scratch), stream or None),
           "dnnops_layernorm_backward")


def layernorm_backward_noalloc_max_scratch_bytes() -> int:
    return int(load().dnnops_layernorm_backward_noalloc_max_scratch_bytes())


def layernorm_backward_noalloc(x, dy, gamma, mean, rstd, rows: int, cols: int, dx, dgamma, dbeta,
                               stream: int = 0) -> None:
    _check(load().dnnops_layernorm_backward_noalloc(_ptr(x), _ptr(dy), _ptr(gamma), _ptr(mean),
                                                    _ptr(rstd), rows, cols, _ptr(dx), _ptr(dgamma),
                                                    _ptr(dbeta), stream or None),
           "dnnops_layernorm_backward_noalloc")


def softmax_forward(x, y, rows: int, cols: int, stream: int = 0) -> None:
    _check(load().dnnops_softmax_forward(_ptr(x), _ptr(y), rows, cols, stream or None),
           "dnnops_softmax_forward")


def softmax_backward(y, dy, dx, rows: int, cols: int, stream: int = 0) -> None:
    _check(load().dnnops_softmax_backward(_ptr(y), _ptr(dy), _ptr(dx), rows, cols, stream or None),
           "dnnops_softmax_backward")

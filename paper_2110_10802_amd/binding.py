"""ctypes binding of libmbconv (argument marshalling only).

The functions mirror include/mbconv.h one to one.  Tensors are anything with a
``data_ptr()`` method (PyTorch-ROCm tensors are used for device memory and the
stream; nothing is computed in Python).  There is no fallback: if the HIP
library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Any, Dict, Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmbconv.so")

MBCONV_F32, MBCONV_BF16 = 0, 1
MBCONV_RECOMPUTE, MBCONV_STORE = 0, 1
MBCONV_ACT_SWISH, MBCONV_ACT_RELU6 = 0, 1
ABI_VERSION = 4
ABSENT = C.c_size_t(-1).value

PARAM_NAMES = ["w_expand", "bn1_gamma", "bn1_beta", "w_dw", "bn2_gamma", "bn2_beta", "se_w1",
               "se_b1", "se_w2", "se_b2", "w_proj", "bn3_gamma", "bn3_beta"]
RUNNING_NAMES = ["bn1_mean", "bn1_var", "bn2_mean", "bn2_var", "bn3_mean", "bn3_var"]
SAVED_NAMES = ["e", "d", "p", "bn1", "bn2", "bn3", "z", "g", "q", "a1", "sc"]
EXPORTS = ["mbconv_workspace_size", "mbconv_saved_offsets", "mbconv_forward", "mbconv_backward",
           "mbconv_forward_probed", "mbconv_backward_probed", "mbconv_eval_workspace_size",
           "mbconv_forward_eval", "mbconv_forward_eval_probed", "mbconv_step_engine",
           "mbconv_status_string", "mbconv_abi_version"]
# mbconv_engine values
ENGINES = {0: "vector", 1: "mfma_f32", 2: "mfma_bf16", 3: "mfma_bf16x3"}
# mbconv_step values (launch order of the two calls)
STEPS = {"expand_conv": 1, "bn1_finalize": 2, "dw_fwd": 3, "bn2_finalize": 4, "se_pool": 5,
         "se_fc": 6, "proj_conv": 7, "bn3_finalize": 8, "bn3_apply": 9, "bn3_bwd_reduce": 10,
         "bn3_bwd_finalize": 11, "proj_dgrad": 12, "proj_wgrad": 13, "gate_sums": 14, "se_bwd": 15,
         "dw_bwd": 16, "dw_wgrad_reduce": 17, "bn1_bwd_finalize": 18, "expand_dgrad": 19,
         "expand_wgrad": 20}
FORWARD_STEPS = [n for n, v in STEPS.items() if v <= 9]


class MBConvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class Desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("N", "Cin", "H", "W", "Cexp", "Cse", "Cout", "k", "stride",
                                          "pad", "has_expand", "residual", "dtype", "policy")] + \
               [("bn_eps", C.c_float), ("bn_momentum", C.c_float), ("activation", C.c_int32),
                ("no_se", C.c_int32)]


class Params(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in PARAM_NAMES]


class Grads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in PARAM_NAMES]


class BNState(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in RUNNING_NAMES]


class Probe(C.Structure):
    _fields_ = [("step", C.c_int32), ("start_event", C.c_void_p), ("stop_event", C.c_void_p)]


class SavedLayout(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in SAVED_NAMES]


_lib = None


def load() -> C.CDLL:
    """Load libmbconv.so; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2110_10802_amd.build` "
                "(there is no CPU or PyTorch fallback)")
        lib = C.CDLL(LIB_PATH)
        vp = C.c_void_p
        lib.mbconv_abi_version.restype = C.c_int32
        lib.mbconv_status_string.restype = C.c_char_p
        lib.mbconv_status_string.argtypes = [C.c_int]
        lib.mbconv_workspace_size.restype = C.c_int
        lib.mbconv_workspace_size.argtypes = [C.POINTER(Desc), C.POINTER(C.c_size_t),
                                              C.POINTER(C.c_size_t)]
        lib.mbconv_saved_offsets.restype = C.c_int
        lib.mbconv_saved_offsets.argtypes = [C.POINTER(Desc), C.POINTER(SavedLayout)]
        lib.mbconv_forward.restype = C.c_int
        lib.mbconv_forward.argtypes = [C.POINTER(Desc), C.POINTER(Params), C.POINTER(BNState), vp,
                                       vp, vp, vp, vp]
        lib.mbconv_backward.restype = C.c_int
        lib.mbconv_backward.argtypes = [C.POINTER(Desc), C.POINTER(Params), vp, vp, vp, vp, vp,
                                        C.POINTER(Grads), vp]
        lib.mbconv_forward_probed.restype = C.c_int
        lib.mbconv_forward_probed.argtypes = lib.mbconv_forward.argtypes + [C.POINTER(Probe)]
        lib.mbconv_backward_probed.restype = C.c_int
        lib.mbconv_backward_probed.argtypes = lib.mbconv_backward.argtypes + [C.POINTER(Probe)]
        lib.mbconv_eval_workspace_size.restype = C.c_int
        lib.mbconv_eval_workspace_size.argtypes = [C.POINTER(Desc), C.POINTER(C.c_size_t)]
        lib.mbconv_forward_eval.restype = C.c_int
        lib.mbconv_forward_eval.argtypes = [C.POINTER(Desc), C.POINTER(Params), C.POINTER(BNState),
                                            vp, vp, vp, vp]
        lib.mbconv_forward_eval_probed.restype = C.c_int
        lib.mbconv_forward_eval_probed.argtypes = lib.mbconv_forward_eval.argtypes + [C.POINTER(Probe)]
        if lib.mbconv_abi_version() != ABI_VERSION:
            raise RuntimeError("libmbconv.so ABI version mismatch; rebuild")
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().mbconv_status_string(int(status)).decode()


def _ptr(t: Any) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return int(t.data_ptr())


def make_desc(shape: Any, policy: int = MBCONV_RECOMPUTE) -> Desc:
    """Descriptor from any object with the BlockShape attributes."""
    return Desc(shape.N, shape.Cin, shape.H, shape.W, shape.Cexp, shape.Cse, shape.Cout, shape.k,
                shape.stride, shape.pad, int(shape.has_expand), int(shape.residual),
                MBCONV_BF16 if shape.dtype == "bf16" else MBCONV_F32, int(policy),
                float(shape.eps), float(shape.momentum),
                MBCONV_ACT_RELU6 if getattr(shape, "activation", "swish") == "relu6" else MBCONV_ACT_SWISH,
                0 if getattr(shape, "has_se", True) else 1)


def _fill(struct, tensors: Optional[Dict[str, Any]]):
    if tensors is not None:
        for name, _ in struct._fields_:
            setattr(struct, name, _ptr(tensors.get(name)))
    return struct


def mbconv_workspace_size(desc: Desc) -> Tuple[int, int]:
    saved, scratch = C.c_size_t(0), C.c_size_t(0)
    rc = load().mbconv_workspace_size(C.byref(desc), C.byref(saved), C.byref(scratch))
    if rc != 0:
        raise MBConvError(rc, "mbconv_workspace_size")
    return saved.value, scratch.value


def mbconv_saved_offsets(desc: Desc) -> Dict[str, Optional[int]]:
    lay = SavedLayout()
    rc = load().mbconv_saved_offsets(C.byref(desc), C.byref(lay))
    if rc != 0:
        raise MBConvError(rc, "mbconv_saved_offsets")
    return {n: (None if getattr(lay, n) == ABSENT else getattr(lay, n)) for n in SAVED_NAMES}


def mbconv_forward(desc: Desc, params: Dict[str, Any], running: Optional[Dict[str, Any]], x: Any,
                   out: Any, saved_ws: Any, scratch_ws: Any, stream: int = 0) -> None:
    mbconv_forward_probed(desc, params, running, x, out, saved_ws, scratch_ws, stream, None)


def mbconv_backward(desc: Desc, params: Dict[str, Any], x: Any, dout: Any, saved_ws: Any,
                    scratch_ws: Any, dx: Any, grads: Dict[str, Any], stream: int = 0) -> None:
    mbconv_backward_probed(desc, params, x, dout, saved_ws, scratch_ws, dx, grads, stream, None)


def mbconv_forward_probed(desc: Desc, params: Any, running: Any, x: Any, out: Any, saved_ws: Any,
                          scratch_ws: Any, stream: int = 0, probe: Optional[Probe] = None) -> None:
    """``params`` / ``running`` may be dicts of tensors or already filled structs."""
    ps = params if isinstance(params, Params) else _fill(Params(), params)
    rs = running if isinstance(running, BNState) or running is None else _fill(BNState(), running)
    lib = load()
    if probe is None:
        rc = lib.mbconv_forward(C.byref(desc), C.byref(ps), C.byref(rs) if rs is not None else None,
                                _ptr(x), _ptr(out), _ptr(saved_ws), _ptr(scratch_ws), stream or None)
    else:
        rc = lib.mbconv_forward_probed(C.byref(desc), C.byref(ps),
                                       C.byref(rs) if rs is not None else None, _ptr(x), _ptr(out),
                                       _ptr(saved_ws), _ptr(scratch_ws), stream or None,
                                       C.byref(probe))
    if rc != 0:
        raise MBConvError(rc, "mbconv_forward")


def mbconv_step_engine(desc: Desc, step: int) -> int:
    """Arithmetic units that serve one step of the launch sequence (host only): key of ENGINES."""
    eng = C.c_int32(0)
    rc = load().mbconv_step_engine(C.byref(desc), int(step), C.byref(eng))
    if rc != 0:
        raise MBConvError(rc, "mbconv_step_engine")
    return eng.value


def mbconv_eval_workspace_size(desc: Desc) -> int:
    nbytes = C.c_size_t(0)
    rc = load().mbconv_eval_workspace_size(C.byref(desc), C.byref(nbytes))
    if rc != 0:
        raise MBConvError(rc, "mbconv_eval_workspace_size")
    return nbytes.value


def mbconv_forward_eval(desc: Desc, params: Any, running: Any, x: Any, out: Any, workspace: Any,
                        stream: int = 0) -> None:
    mbconv_forward_eval_probed(desc, params, running, x, out, workspace, stream, None)


def mbconv_forward_eval_probed(desc: Desc, params: Any, running: Any, x: Any, out: Any,
                               workspace: Any, stream: int = 0,
                               probe: Optional[Probe] = None) -> None:
    ps = params if isinstance(params, Params) else _fill(Params(), params)
    rs = running if isinstance(running, BNState) or running is None else _fill(BNState(), running)
    lib = load()
    rsp = C.byref(rs) if rs is not None else None
    if probe is None:
        rc = lib.mbconv_forward_eval(C.byref(desc), C.byref(ps), rsp, _ptr(x), _ptr(out),
                                     _ptr(workspace), stream or None)
    else:
        rc = lib.mbconv_forward_eval_probed(C.byref(desc), C.byref(ps), rsp, _ptr(x), _ptr(out),
                                            _ptr(workspace), stream or None, C.byref(probe))
    if rc != 0:
        raise MBConvError(rc, "mbconv_forward_eval")


def mbconv_backward_probed(desc: Desc, params: Any, x: Any, dout: Any, saved_ws: Any,
                           scratch_ws: Any, dx: Any, grads: Any, stream: int = 0,
                           probe: Optional[Probe] = None) -> None:
    ps = params if isinstance(params, Params) else _fill(Params(), params)
    gs = grads if isinstance(grads, Grads) else _fill(Grads(), grads)
    lib = load()
    if probe is None:
        rc = lib.mbconv_backward(C.byref(desc), C.byref(ps), _ptr(x), _ptr(dout), _ptr(saved_ws),
                                 _ptr(scratch_ws), _ptr(dx), C.byref(gs), stream or None)
    else:
        rc = lib.mbconv_backward_probed(C.byref(desc), C.byref(ps), _ptr(x), _ptr(dout),
                                        _ptr(saved_ws), _ptr(scratch_ws), _ptr(dx), C.byref(gs),
                                        stream or None, C.byref(probe))
    if rc != 0:
        raise MBConvError(rc, "mbconv_backward")

"""Host-only checks of the C ABI: the library loads, exports every symbol the header
declares, and rejects bad arguments before touching the GPU.  No compute call is made."""
import ctypes as C
import os
import re

import pytest

from mbconv_inputs import CONFIG0, CONFIG1, CONFIG3, b0_chain
from paper_2110_10802_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "mbconv.h")).read()
    declared = set(re.findall(r"\b(mbconv_[a-z_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)
    lib = B.load()
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.mbconv_abi_version() == B.ABI_VERSION


def test_library_exports_every_dnnops_symbol():
    from paper_2110_10802_amd import dnnops as D
    hdr = open(os.path.join(ROOT, "include", "dnnops.h")).read()
    declared = set(re.findall(r"\b(dnnops_[a-z_]+)\s*\(", hdr))
    assert declared == set(D.EXPORTS), declared ^ set(D.EXPORTS)
    lib = D.load()
    for name in declared:
        assert hasattr(lib, name), name
    assert int(re.search(r"#define DNNOPS_MAX_COLS (\d+)", hdr).group(1)) == D.MAX_COLS
    # host-side argument checks: nothing reaches the GPU
    assert lib.dnnops_mish_forward(None, None, 16, None) == -1
    assert lib.dnnops_mish_forward(16, 32, 0, None) == -1
    assert lib.dnnops_mish_forward(16, 36, 8, None) == -4
    assert lib.dnnops_softmax_forward(16, 32, 4, D.MAX_COLS + 1, None) == -2
    assert lib.dnnops_softmax_forward(16, 32, 0, 8, None) == -1
    assert lib.dnnops_layernorm_forward(16, 32, 48, -1.0, 4, 8, 64, 80, 96, None) == -1
    assert D.layernorm_backward_scratch_bytes(0, 8) == 0
    assert D.layernorm_backward_scratch_bytes(4096, 1024) == 2 * 256 * 1024 * 4
    assert D.layernorm_backward_scratch_bytes(100000, 1024) == 2 * 512 * 1024 * 4
    # the entry point without a workspace argument: its size limit is checked on the host
    assert D.layernorm_backward_noalloc_max_scratch_bytes() == 8 << 20
    assert lib.dnnops_layernorm_backward_noalloc(16, 32, 48, 64, 80, 100000, 8192, 96, 112, 128, None) == -3
    assert lib.dnnops_layernorm_backward_noalloc(16, 32, 48, 64, 80, 0, 8, 96, 112, 128, None) == -1
    assert lib.dnnops_layernorm_backward_noalloc(16, 36, 48, 64, 80, 4, 8, 96, 112, 128, None) == -4


def test_status_strings():
    assert B.status_string(0) == "ok"
    for code in (-1, -2, -3, -4, -5):
        assert B.status_string(code) not in ("ok", "unknown status")
    assert B.status_string(-99) == "unknown status"


def test_workspace_sizes_cover_the_saved_tensors():
    for s in [CONFIG0, CONFIG1, CONFIG3] + b0_chain():
        d = B.make_desc(s)
        saved, scratch = B.mbconv_workspace_size(d)
        esz = 2 if s.dtype == "bf16" else 4
        need = esz * s.N * (s.Cexp * s.Ho * s.Wo + s.Cout * s.Ho * s.Wo)
        if s.has_expand:
            need += esz * s.N * s.Cexp * s.H * s.W
        # fp32 wide blocks also keep bf16-plane images of the two 1x1 conv weights, in both
        # orientations (6 bytes per element and orientation, tiles of 64 x 32)
        up = lambda v, m: (v + m - 1) // m * m
        images = 6 * (up(s.Cexp, 64) * up(s.Cin, 32) + up(s.Cout, 64) * up(s.Cexp, 32)
                      + up(s.Cexp, 64) * up(s.Cout, 32) + up(s.Cin, 64) * up(s.Cexp, 32))
        assert saved >= need and saved < need * 1.05 + (1 << 20) + images
        assert scratch > 0
        lay = B.mbconv_saved_offsets(d)
        assert (lay["e"] is None) == (not s.has_expand)
        assert lay["a1"] is None and lay["sc"] is None
        offs = sorted(v for v in lay.values() if v is not None)
        assert all(o % 256 == 0 for o in offs) and len(set(offs)) == len(offs)
        saved_store, _ = B.mbconv_workspace_size(B.make_desc(s, B.MBCONV_STORE))
        assert saved_store > saved
        assert B.mbconv_saved_offsets(B.make_desc(s, B.MBCONV_STORE))["sc"] is not None


def _bad(**kw):
    d = B.make_desc(CONFIG0)
    for k, v in kw.items():
        setattr(d, k, v)
    return d


@pytest.mark.parametrize("kw,code", [
    (dict(N=0), -1), (dict(Cexp=0), -1), (dict(dtype=7), -1), (dict(policy=3), -1),
    (dict(has_expand=0), -1),            # Cexp != Cin without an expansion conv
    (dict(residual=1, stride=2), -1),    # residual needs stride 1
    (dict(residual=1, Cout=24), -1),     # ... and Cin == Cout
    (dict(bn_eps=-1.0), -1), (dict(bn_momentum=2.0), -1),
    (dict(k=7, pad=3), -2), (dict(stride=3, residual=0), -2), (dict(pad=0), -2),
    (dict(H=200), -2),
])
def test_descriptor_validation(kw, code):
    with pytest.raises(B.MBConvError) as ei:
        B.mbconv_workspace_size(_bad(**kw))
    assert ei.value.status == code


def test_forward_backward_reject_bad_pointers_on_the_host():
    # every check below fails before the first launch, so no GPU is needed
    d = B.make_desc(CONFIG0)
    good = 4096  # an aligned, never dereferenced address
    params = {n: good for n in B.PARAM_NAMES}
    running = {n: good for n in B.RUNNING_NAMES}
    with pytest.raises(B.MBConvError) as ei:
        B.mbconv_forward(d, params, running, None, good, good, good)
    assert ei.value.status == -1
    with pytest.raises(B.MBConvError) as ei:
        B.mbconv_forward(d, dict(params, w_proj=None), running, good, good, good, good)
    assert ei.value.status == -1
    with pytest.raises(B.MBConvError) as ei:
        B.mbconv_forward(d, params, running, good + 4, good, good, good)
    assert ei.value.status == -4
    with pytest.raises(B.MBConvError) as ei:
        B.mbconv_forward(d, dict(params, se_w1=good + 8), running, good, good, good, good)
    assert ei.value.status == -4
    with pytest.raises(B.MBConvError) as ei:
        B.mbconv_forward(d, params, dict(running, bn3_var=None), good, good, good, good)
    assert ei.value.status == -1
    grads = {n: good for n in B.PARAM_NAMES}
    with pytest.raises(B.MBConvError) as ei:
        B.mbconv_backward(d, params, good, good, good, good, None, grads)
    assert ei.value.status == -1
    with pytest.raises(B.MBConvError) as ei:
        B.mbconv_backward(d, params, good, good, good, good, good, dict(grads, w_dw=None))
    assert ei.value.status == -1
    with pytest.raises(B.MBConvError) as ei:
        B.mbconv_backward(d, params, good, good + 2, good, good, good, grads)
    assert ei.value.status == -4
    lib = B.load()
    assert lib.mbconv_forward(None, None, None, None, None, None, None, None) == -1
    assert lib.mbconv_workspace_size(C.byref(d), None, None) == -1


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2110_10802_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, f)


def test_step_engine_query():
    """Host-only query: which units serve a step (used by bench.py to price its GEMM figures)."""
    chain = b0_chain()
    E = B.ENGINES
    # block 10 (112 -> 672 -> 112, 14x14, fp32): all six 1x1 steps on bf16 MFMAs over split operands
    d = B.make_desc(chain[9])
    for name in ("expand_conv", "proj_conv", "proj_dgrad", "proj_wgrad", "expand_dgrad", "expand_wgrad"):
        assert E[B.mbconv_step_engine(d, B.STEPS[name])] == "mfma_bf16x3", name
    assert E[B.mbconv_step_engine(d, B.STEPS["dw_fwd"])] == "vector"
    # block 14 (7x7): the convolutions use plane tiles, the weight gradients the fp32 MFMA kernels
    d = B.make_desc(chain[13])
    assert E[B.mbconv_step_engine(d, B.STEPS["proj_conv"])] == "mfma_bf16x3"
    assert E[B.mbconv_step_engine(d, B.STEPS["proj_wgrad"])] == "mfma_f32"
    # config 1 (24 -> 144 -> 24): skinny kernels on the fp32 MFMA; the fused backward kernels make
    # the weight-gradient steps plain sums
    d = B.make_desc(CONFIG1)
    assert E[B.mbconv_step_engine(d, B.STEPS["expand_conv"])] == "mfma_f32"
    assert E[B.mbconv_step_engine(d, B.STEPS["expand_dgrad"])] == "mfma_f32"
    assert E[B.mbconv_step_engine(d, B.STEPS["expand_wgrad"])] == "vector"
    # config 3 (bf16 storage)
    d = B.make_desc(CONFIG3)
    assert E[B.mbconv_step_engine(d, B.STEPS["proj_conv"])] == "mfma_bf16"
    assert E[B.mbconv_step_engine(d, B.STEPS["expand_wgrad"])] == "mfma_bf16"
    with pytest.raises(B.MBConvError):
        B.mbconv_step_engine(d, 0)
    with pytest.raises(B.MBConvError):
        B.mbconv_step_engine(d, 99)


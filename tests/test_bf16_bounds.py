"""Where the bf16 parity bounds come from, shown on the CPU with the oracle alone (no HIP code
is involved in anything here).

The benchmark states "max relative error <= 2e-2" for bf16 storage.  These tests fix, for the
shape of benchmark config 3 (112 -> 672 -> 112 channels, 14x14, 5x5 depthwise, batch >= 16):

  1. an fp64 computation that does nothing but store its activation-sized tensors as bf16
     already leaves 2e-2 under the element-wise metric max_i |err_i| / max(|ref_i|, rms(ref)),
     so that metric at 2e-2 cannot be met by any bf16-storage implementation, while under
     max|err| / max|ref| the same computation stays below 1.5e-2: the GPU-versus-oracle bf16
     tests therefore use the second metric at 2e-2 (parity_util.TOL, metric_for);
  2. rounding the operands of the 1x1 convolutions to bf16 as well (what the bf16 matrix-core
     kernels do) costs at most a few 1e-3 more under either metric;
  3. the element-wise metric is applied against the same computation with the roundings in
     place (tests/rounding_model.py); there, noise of fp32 size ahead of the roundings moves
     BN1's gamma gradient by more than two bf16 ulps (2^-6) at batch 16 but never by four
     (2^-5), and every other tensor by less than 2^-6 + 1e-3: the bounds of
     test_parity_gpu.test_bf16_matches_rounding_model.
"""
import numpy as np
import pytest

from mbconv_inputs import CONFIG3, make_block_inputs
from oracle import oracle as orc
from parity_util import linf_err, rel_err
from rounding_model import rounding_model

BATCH = 16
SEEDS = (0, 5)


def _flat(m):
    return {**{k: v for k, v in m.items() if k != "grads"}, **m["grads"]}


@pytest.fixture(scope="module", params=SEEDS)
def case(request):
    s = CONFIG3.with_batch(BATCH)
    t = make_block_inputs(s, seed=request.param)
    f, b = orc.mbconv_step(s, t)
    ref = {"out": f.out, "e": f.tape["e"], "d": f.tape["d"], "p": f.tape["p"], "dx": b.dx, **b.grads}
    return s, t, ref


def test_storage_rounding_alone_breaks_the_elementwise_bound(case):
    s, t, ref = case
    m = _flat(rounding_model(s, t, storage=True, mfma_bf16=False))
    elem = {k: rel_err(m[k], ref[k]) for k in ref}
    linf = {k: linf_err(m[k], ref[k]) for k in ref}
    print({k: f"{elem[k]:.4f}/{linf[k]:.4f}" for k in ref})
    # BN1's gamma gradient is the small residual of a heavily cancelling sum (BN2 makes the loss
    # almost invariant to the scale of a1): storage rounding alone moves it by about 4e-2
    assert elem["bn1_gamma"] > 3e-2
    assert sum(v > 2e-2 for v in elem.values()) >= 1
    assert max(elem.values()) < 8e-2
    # relative to the tensor's largest magnitude the same model is well inside 2e-2
    assert linf["bn1_gamma"] < 1.5e-2
    assert all(v < 8e-3 for k, v in linf.items() if k != "bn1_gamma"), linf


def test_operand_rounding_costs_little_more(case):
    s, t, ref = case
    a = _flat(rounding_model(s, t, storage=True, mfma_bf16=False))
    b = _flat(rounding_model(s, t, storage=True, mfma_bf16=True))
    for k in ref:
        la, lb = linf_err(a[k], ref[k]), linf_err(b[k], ref[k])
        ea, eb = rel_err(a[k], ref[k]), rel_err(b[k], ref[k])
        assert lb < la + 3e-3, (k, la, lb)
        assert eb < ea + 1.2e-2, (k, ea, eb)
    lb = {k: linf_err(b[k], ref[k]) for k in ref}
    assert lb["bn1_gamma"] < 1.5e-2
    assert all(v < 8e-3 for k, v in lb.items() if k != "bn1_gamma"), lb


def test_fp32_noise_ahead_of_the_roundings_moves_bn1_gamma_beyond_two_ulps(case):
    s, t, _ = case
    base = _flat(rounding_model(s, t, storage=True, mfma_bf16=True))
    spread = {}
    for seed in (1, 2, 3):
        n = _flat(rounding_model(s, t, storage=True, mfma_bf16=True, noise=1e-7, seed=seed))
        for k in base:
            spread.setdefault(k, []).append(rel_err(n[k], base[k]))
    print({k: [f"{v:.4f}" for v in vs] for k, vs in spread.items()})
    two_ulps, four_ulps = 2.0 ** -6, 2.0 ** -5
    # BN1's gamma gradient: beyond two ulps in at least one draw, never beyond four
    assert max(spread["bn1_gamma"]) > two_ulps * 0.85
    assert max(spread["bn1_gamma"]) < four_ulps
    # a stored tensor: one flipped value is one bf16 ulp (at most 2^-7 of it), a flip on top of a
    # propagated flip two; the parameter gradients average the flips out
    for k in ("e", "d", "p", "dx"):
        assert max(spread[k]) <= two_ulps * 1.01, (k, spread[k])
    assert max(spread["out"]) <= two_ulps + 1.5e-3, spread["out"]
    for k in spread:
        if k not in ("out", "e", "d", "p", "dx", "bn1_gamma"):
            assert max(spread[k]) < two_ulps, (k, spread[k])

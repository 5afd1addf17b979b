"""The oracle's steps with bf16 rounding inserted at chosen points, built from the oracle's
own primitives (CPU, fp64 between the roundings).  Test infrastructure only.

Two kinds of rounding points exist in a bf16-storage implementation of the block:
  storage  -- every activation-sized tensor that crosses HBM is stored as bf16: e, d, p, out on
              the way forward, G, dy1, dx on the way back (the reading of "bf16 storage with fp32
              accumulation" for benchmark config 3);
  operands -- where the 1x1 convolutions run on the bf16 matrix cores, their operands are
              rounded to bf16 once after the fp32 prologue: sc = act(BN2(d))*gate, dp and de
              (the outputs of BN3's and BN1's backward); accumulation stays fp32.
`noise` multiplies every value about to be rounded by (1 + noise*N(0,1)): the size of fp32
rounding noise ahead of a bf16 rounding, which moves values across rounding boundaries.
"""
from __future__ import annotations

import numpy as np

from mbconv_inputs import round_to_bf16
from oracle import oracle as orc


def rounding_model(s, t, storage=True, mfma_bf16=False, noise=0.0, seed=0):
    rng = np.random.default_rng(seed)

    def _round(a):
        if noise:
            a = a * (1.0 + noise * rng.standard_normal(a.shape))
        return round_to_bf16(a.astype(np.float32)).astype(np.float64)

    rb = _round if storage else (lambda v: v)
    ro = _round if mfma_bf16 else (lambda v: v)

    if getattr(s, "activation", "swish") == "relu6":
        def act(v):
            return np.minimum(np.maximum(v, 0.0), 6.0)

        def act_grad(v):
            return ((v > 0.0) & (v < 6.0)).astype(np.float64)
    else:
        def act(v):
            return v / (1.0 + np.exp(-v))

        def act_grad(v):
            sg = 1.0 / (1.0 + np.exp(-v))
            return sg * (1.0 + v * (1.0 - sg))

    x, dout = t["x"].astype(np.float64), t["dout"].astype(np.float64)
    e = rb(orc.conv1x1(t["w_expand"], x))
    y1, xh1, _, v1, _, _ = orc.bn_fwd(e, t["bn1_gamma"], t["bn1_beta"], s.eps, s.momentum)
    a1 = act(y1)
    d = rb(orc.depthwise_fwd(t["w_dw"], a1, s.stride, s.pad))
    y2, xh2, _, v2, _, _ = orc.bn_fwd(d, t["bn2_gamma"], t["bn2_beta"], s.eps, s.momentum)
    a2 = act(y2)
    has_se = getattr(s, "has_se", True)
    se = orc.se_fwd(a2, t["se_w1"], t["se_b1"], t["se_w2"], t["se_b2"]) if has_se else None
    sc_op = ro(se.sc if has_se else a2)
    p = rb(orc.conv1x1(t["w_proj"], sc_op))
    y3, xh3, _, v3, _, _ = orc.bn_fwd(p, t["bn3_gamma"], t["bn3_beta"], s.eps, s.momentum)
    out = rb(y3 + (x if s.residual else 0.0))
    dp, dg3, db3 = orc.bn_bwd(dout, xh3, t["bn3_gamma"], v3, s.eps)
    dp_op = ro(dp)
    G = rb(orc.conv1x1_bwd_input(t["w_proj"], dp_op))
    g = {"w_proj": orc.conv1x1_bwd_weight(sc_op, dp_op), "bn3_gamma": dg3, "bn3_beta": db3}
    if has_se:
        sb = orc.se_bwd(a2, t["se_w1"], t["se_w2"], se, G)
        g.update(se_w1=sb.dw1, se_b1=sb.db1, se_w2=sb.dw2, se_b2=sb.db2)
        da2 = sb.da2
    else:
        da2 = G
    dd, g["bn2_gamma"], g["bn2_beta"] = orc.bn_bwd(da2 * act_grad(y2), xh2, t["bn2_gamma"], v2, s.eps)
    g["w_dw"] = orc.depthwise_bwd_weight(a1, dd, s.k, s.stride, s.pad)
    da1 = orc.depthwise_bwd_input(t["w_dw"], dd, s.H, s.W, s.stride, s.pad)
    dy1 = rb(da1 * act_grad(y1))
    de, g["bn1_gamma"], g["bn1_beta"] = orc.bn_bwd(dy1, xh1, t["bn1_gamma"], v1, s.eps)
    de_op = ro(de)
    g["w_expand"] = orc.conv1x1_bwd_weight(x, de_op)
    dx = rb(orc.conv1x1_bwd_input(t["w_expand"], de_op) + (dout if s.residual else 0.0))
    return {"out": out, "e": e, "d": d, "p": p, "dx": dx, "grads": g}

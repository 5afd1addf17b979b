"""Seeded synthetic inputs and block shapes for the MBConv training step.

This module serves both the CPU oracle's tests and the HIP path's tests and
benchmark.  It holds no arithmetic of the method: only shapes, random draws and
the rounding of inputs to bf16 storage.

Recipe (one ``numpy.random.default_rng(seed)`` stream per block, fixed draw
order x, W_e, gamma1, beta1, w_dw, gamma2, beta2, W1, b1, W2, b2, W_p, gamma3,
beta3, dOut):
  x, dOut ~ N(0,1); conv / FC weights Kaiming-normal, std = sqrt(2/fan_in) with
  fan_in = Cin (W_e), k*k (w_dw), Cexp (W_p, W1), Cse (W2);
  BN gamma = 1 + 0.1 N(0,1), beta = 0.1 N(0,1); SE biases 0.1 N(0,1);
  running mean 0, running variance 1.
The shapes are those of EfficientNet-B0's MBConv blocks (and one MobileNet-V2 block); the
values stand in for the ImageNet activations and trained weights the paper's measurement ran on.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List

import numpy as np

BN_EPS = 1e-3
BN_MOMENTUM = 0.01


@dataclass(frozen=True)
class BlockShape:
    N: int
    Cin: int
    H: int
    W: int
    Cexp: int
    Cse: int
    Cout: int
    k: int
    stride: int
    has_expand: bool = True
    residual: bool = False
    dtype: str = "f32"  # activation / conv-weight storage: "f32" or "bf16"
    eps: float = BN_EPS
    momentum: float = BN_MOMENTUM
    activation: str = "swish"  # "swish" (EfficientNet MBConv) or "relu6" (MobileNet-V2 block)
    has_se: bool = True        # False: no squeeze-and-excitation stage (Cse is ignored)

    @property
    def pad(self) -> int:
        return (self.k - 1) // 2

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad - self.k) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad - self.k) // self.stride + 1

    def with_batch(self, n: int) -> "BlockShape":
        return replace(self, N=n)


# The five benchmark configurations (single blocks 0-3, the B0 chain is 4).
CONFIG0 = BlockShape(N=2, Cin=16, H=16, W=16, Cexp=96, Cse=4, Cout=16, k=3, stride=1,
                     residual=True)
CONFIG1 = BlockShape(N=32, Cin=24, H=56, W=56, Cexp=144, Cse=6, Cout=24, k=3, stride=1,
                     residual=True)
CONFIG2 = BlockShape(N=64, Cin=24, H=56, W=56, Cexp=144, Cse=6, Cout=40, k=5, stride=2,
                     residual=False)
CONFIG3 = BlockShape(N=128, Cin=112, H=14, W=14, Cexp=672, Cse=28, Cout=112, k=5, stride=1,
                     residual=True, dtype="bf16")

# (kernel, expand ratio, out channels, stride of first repeat, repeats)
_B0_STAGES = [(3, 1, 16, 1, 1), (3, 6, 24, 2, 2), (5, 6, 40, 2, 2), (3, 6, 80, 2, 3),
              (5, 6, 112, 1, 3), (5, 6, 192, 2, 4), (3, 6, 320, 1, 1)]


def b0_chain(N: int = 64, Cin: int = 32, H: int = 112, dtype: str = "f32") -> List[BlockShape]:
    """The 16 MBConv blocks of EfficientNet-B0 as a chain of shapes."""
    blocks = []
    c, h = Cin, H
    for k, ratio, cout, stride, reps in _B0_STAGES:
        for rep in range(reps):
            s = stride if rep == 0 else 1
            b = BlockShape(N=N, Cin=c, H=h, W=h, Cexp=c * ratio, Cse=max(1, c // 4), Cout=cout,
                           k=k, stride=s, has_expand=(ratio != 1),
                           residual=(s == 1 and c == cout), dtype=dtype)
            blocks.append(b)
            c, h = cout, b.Ho
    return blocks



# MobileNet-V2 inverted-residual block (ReLU6, no squeeze-and-excitation), the network the paper
# also times: the stride-1 repeat of its 56x56 stage (24 -> 144 -> 24, 3x3), batch 32 -- the same
# tensor shapes as config 1, so the two activations can be compared kernel by kernel.
MBV2_BLOCK = BlockShape(N=32, Cin=24, H=56, W=56, Cexp=144, Cse=1, Cout=24, k=3, stride=1,
                        residual=True, activation="relu6", has_se=False)

# 0-3: the single-block benchmark configurations; 5: the MobileNet-V2 block (4 is the chain)
CONFIGS = {0: CONFIG0, 1: CONFIG1, 2: CONFIG2, 3: CONFIG3, 5: MBV2_BLOCK}


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16) << 16
    out = r.astype(np.uint32).view(np.float32)
    return np.where(np.isfinite(a), out, a).astype(np.float32)


PARAM_NAMES = ["w_expand", "bn1_gamma", "bn1_beta", "w_dw", "bn2_gamma", "bn2_beta", "se_w1",
               "se_b1", "se_w2", "se_b2", "w_proj", "bn3_gamma", "bn3_beta"]
# tensors stored in the activation dtype (rounded to bf16 for the bf16 config)
STORAGE_DTYPE_NAMES = ["x", "dout", "w_expand", "w_dw", "w_proj"]


def make_block_inputs(s: BlockShape, seed: int = 0, with_x: bool = True,
                      with_dout: bool = True) -> Dict[str, np.ndarray]:
    """All inputs of one block as fp32 numpy arrays (bf16-rounded where stored as bf16)."""
    rng = np.random.default_rng(seed)
    f32 = np.float32

    def normal(shape, std=1.0, mean=0.0):
        return (mean + std * rng.standard_normal(shape, dtype=np.float64)).astype(f32)

    t: Dict[str, np.ndarray] = {}
    x = normal((s.N, s.Cin, s.H, s.W))
    if with_x:
        t["x"] = x
    if s.has_expand:
        t["w_expand"] = normal((s.Cexp, s.Cin), np.sqrt(2.0 / s.Cin))
        t["bn1_gamma"] = normal((s.Cexp,), 0.1, 1.0)
        t["bn1_beta"] = normal((s.Cexp,), 0.1)
    else:
        # the draws are made anyway so later tensors do not depend on has_expand
        normal((s.Cexp, s.Cin))
        normal((s.Cexp,))
        normal((s.Cexp,))
    t["w_dw"] = normal((s.Cexp, s.k, s.k), np.sqrt(2.0 / (s.k * s.k)))
    t["bn2_gamma"] = normal((s.Cexp,), 0.1, 1.0)
    t["bn2_beta"] = normal((s.Cexp,), 0.1)
    se = {"se_w1": normal((s.Cse, s.Cexp), np.sqrt(2.0 / s.Cexp)), "se_b1": normal((s.Cse,), 0.1),
          "se_w2": normal((s.Cexp, s.Cse), np.sqrt(2.0 / s.Cse)), "se_b2": normal((s.Cexp,), 0.1)}
    if s.has_se:  # (the draws are made anyway so later tensors do not depend on has_se)
        t.update(se)
    t["w_proj"] = normal((s.Cout, s.Cexp), np.sqrt(2.0 / s.Cexp))
    t["bn3_gamma"] = normal((s.Cout,), 0.1, 1.0)
    t["bn3_beta"] = normal((s.Cout,), 0.1)
    dout = normal((s.N, s.Cout, s.Ho, s.Wo))
    if with_dout:
        t["dout"] = dout
    if s.dtype == "bf16":
        for name in STORAGE_DTYPE_NAMES:
            if name in t:
                t[name] = round_to_bf16(t[name])
    for i in (1, 2):
        t[f"bn{i}_mean"] = np.zeros((s.Cexp,), f32)
        t[f"bn{i}_var"] = np.ones((s.Cexp,), f32)
    t["bn3_mean"] = np.zeros((s.Cout,), f32)
    t["bn3_var"] = np.ones((s.Cout,), f32)
    return t

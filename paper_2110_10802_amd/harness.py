"""Device-buffer plumbing around the C ABI for tests, smoke and the benchmark.

PyTorch is used for device memory, host<->device copies and the stream handle only;
every step of the MBConv path runs inside libmbconv.
"""
from __future__ import annotations

from typing import Any, Dict, Optional

import numpy as np
import torch

from . import binding as B


def _tdtype(shape) -> torch.dtype:
    return torch.bfloat16 if shape.dtype == "bf16" else torch.float32


STORAGE = ("x", "dout", "w_expand", "w_dw", "w_proj")


class DeviceBlock:
    """One MBConv block's parameters, state, workspaces and outputs on the GPU."""

    def __init__(self, shape, tensors: Dict[str, np.ndarray], policy: int = B.MBCONV_RECOMPUTE,
                 device: str = "cuda:0", scratch: Optional[torch.Tensor] = None):
        self.shape = shape
        self.device = torch.device(device)
        self.desc = B.make_desc(shape, policy)
        self.act = _tdtype(shape)
        self.params: Dict[str, torch.Tensor] = {}
        for n in B.PARAM_NAMES:
            if n in tensors:
                dt = self.act if n in STORAGE else torch.float32
                self.params[n] = torch.from_numpy(np.ascontiguousarray(tensors[n])).to(
                    self.device, dt).contiguous()
        self.running = {}
        for n in B.RUNNING_NAMES:
            if n in tensors and (shape.has_expand or not n.startswith("bn1")):
                self.running[n] = torch.from_numpy(np.ascontiguousarray(tensors[n])).to(
                    self.device, torch.float32).contiguous()
        saved_bytes, scratch_bytes = B.mbconv_workspace_size(self.desc)
        self.saved_bytes, self.scratch_bytes = saved_bytes, scratch_bytes
        self.saved = torch.empty(saved_bytes, dtype=torch.uint8, device=self.device)
        if scratch is None:
            scratch = torch.empty(scratch_bytes, dtype=torch.uint8, device=self.device)
        assert scratch.numel() >= scratch_bytes
        self.scratch = scratch
        s = shape
        self.out = torch.empty((s.N, s.Cout, s.Ho, s.Wo), dtype=self.act, device=self.device)
        self.dx = torch.empty((s.N, s.Cin, s.H, s.W), dtype=self.act, device=self.device)
        self.grads = {n: torch.empty_like(p, dtype=torch.float32) for n, p in self.params.items()}

    def to_device(self, a: np.ndarray) -> torch.Tensor:
        return torch.from_numpy(np.ascontiguousarray(a)).to(self.device, self.act).contiguous()

    def forward(self, x: torch.Tensor, stream: int = 0) -> torch.Tensor:
        B.mbconv_forward(self.desc, self.params, self.running or None, x, self.out, self.saved,
                         self.scratch, stream)
        return self.out

    def forward_eval(self, x: torch.Tensor, stream: int = 0) -> torch.Tensor:
        """Evaluation-mode forward (running statistics, nothing saved)."""
        if getattr(self, "eval_ws", None) is None:
            nbytes = B.mbconv_eval_workspace_size(self.desc)
            self.eval_ws = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        B.mbconv_forward_eval(self.desc, self.params, self.running, x, self.out, self.eval_ws, stream)
        return self.out

    def backward(self, x: torch.Tensor, dout: torch.Tensor, stream: int = 0) -> torch.Tensor:
        B.mbconv_backward(self.desc, self.params, x, dout, self.saved, self.scratch, self.dx,
                          self.grads, stream)
        return self.dx

    def saved_tensor(self, name: str) -> Optional[np.ndarray]:
        """Copy a named tensor out of the saved workspace (for inspection in tests)."""
        off = B.mbconv_saved_offsets(self.desc)[name]
        if off is None:
            return None
        s = self.shape
        shapes = {"e": (s.N, s.Cexp, s.H, s.W), "a1": (s.N, s.Cexp, s.H, s.W),
                  "d": (s.N, s.Cexp, s.Ho, s.Wo), "sc": (s.N, s.Cexp, s.Ho, s.Wo),
                  "p": (s.N, s.Cout, s.Ho, s.Wo), "bn1": (4, s.Cexp), "bn2": (4, s.Cexp),
                  "bn3": (4, s.Cout), "z": (s.N, s.Cexp), "g": (s.N, s.Cexp), "q": (s.N, s.Cse)}
        shp = shapes[name]
        dt = self.act if name in ("e", "a1", "d", "sc", "p") else torch.float32
        nbytes = int(np.prod(shp)) * (2 if dt == torch.bfloat16 else 4)
        return self.saved[off:off + nbytes].view(dt).reshape(shp).float().cpu().numpy()


def to_numpy(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()

"""Device-buffer plumbing around the binding: uploads one batch with torch, owns outputs and
workspaces, and calls the C entry points.  No head arithmetic happens here."""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as lsr
from .inputs import HeadInputs


class DeviceHead:
    def __init__(self, inp: HeadInputs, *, device: str = "cuda:0", want_index: bool = True,
                 want_backward: Optional[bool] = None, mask: Optional[np.ndarray] = None):
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the HIP path has no CPU fallback")
        lsr.load_library()
        w = inp.workload
        self.B, self.S, self.D, self.V = w.B, w.S, w.D, w.V
        self.dt = lsr.LSR_BF16 if w.dtype == "bf16" else lsr.LSR_F32
        dev = torch.device(device)
        self.dev = dev
        if w.dtype == "bf16":
            self.H = torch.from_numpy(inp.H_bits.view(np.int16)).to(dev).view(torch.bfloat16)
            self.W = torch.from_numpy(inp.W_bits.view(np.int16)).to(dev).view(torch.bfloat16)
        else:
            self.H = torch.from_numpy(inp.H).to(dev)
            self.W = torch.from_numpy(inp.W).to(dev)
        self.bias = torch.from_numpy(inp.bias).to(dev)
        self.mask = torch.from_numpy(np.ascontiguousarray(inp.mask if mask is None else mask, dtype=np.uint8)).to(dev)
        self.Y = torch.empty((self.B, self.V), dtype=torch.float32, device=dev)
        self.I = torch.empty((self.B, self.V), dtype=torch.int32, device=dev) if want_index else None
        self.ws_fwd = torch.empty(lsr.lsr_head_workspace_bytes(self.B, self.S, self.D, self.V, self.dt, False),
                                  dtype=torch.uint8, device=dev)
        bwd = (inp.dY is not None) if want_backward is None else want_backward
        self.has_backward = bwd
        if bwd:
            self.dY = torch.from_numpy(inp.dY).to(dev)
            self.dH = torch.empty((self.B, self.S, self.D), dtype=torch.float32, device=dev)
            self.dW = torch.empty((self.V, self.D), dtype=torch.float32, device=dev)
            self.db = torch.empty((self.V,), dtype=torch.float32, device=dev)
            self.ws_bwd = torch.empty(lsr.lsr_head_workspace_bytes(self.B, self.S, self.D, self.V, self.dt, True),
                                      dtype=torch.uint8, device=dev)

    def _shape(self):
        return (self.B, self.S, self.D, self.V, self.dt)

    def forward(self):
        lsr.lsr_head_forward(*self._shape(), self.H, self.W, self.bias, self.mask, self.Y, self.I, self.ws_fwd)

    def backward(self):
        lsr.lsr_head_backward(*self._shape(), self.H, self.W, self.dY, self.Y, self.I, self.dH, self.dW, self.db,
                              self.ws_bwd)

    def forward_profiled(self):
        return lsr.lsr_head_forward_profiled(*self._shape(), self.H, self.W, self.bias, self.mask, self.Y, self.I,
                                             self.ws_fwd)

    def backward_profiled(self):
        return lsr.lsr_head_backward_profiled(*self._shape(), self.H, self.W, self.dY, self.Y, self.I, self.dH,
                                              self.dW, self.db, self.ws_bwd)

    def poison_outputs(self):
        """Fill every output with NaN so that a test notices anything left unwritten."""
        self.Y.fill_(float("nan"))
        if self.I is not None:
            self.I.fill_(-7)
        if self.has_backward:
            self.dH.fill_(float("nan"))
            self.dW.fill_(float("nan"))
            self.db.fill_(float("nan"))

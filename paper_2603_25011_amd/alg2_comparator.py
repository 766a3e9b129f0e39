"""Benchmark comparator, not part of the product path: the paper's hybrid forward (Sec. 3, Alg. 2).

Per tile of the vocabulary a library GEMM (torch.mm, i.e. hipBLASLt) writes the tile's logits for the
packed valid tokens to memory, then a small hand-written HIP kernel (csrc/alg2_reduce.hip, the paper's
reduce kernel) takes the maximum and arg-max over each sequence and applies bias, ReLU and log1p.
bench.py times this on the workload's own H and W beside the fused kernel and checks its output against
the oracle on a sample.  The product never calls anything in this module.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libalg2_reduce.so")
_lib = None


def load_library():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(f"{_LIB_PATH} is missing: run `python -m paper_2603_25011_amd.build`")
        lib = ctypes.CDLL(_LIB_PATH)
        vp, i64 = ctypes.c_void_p, ctypes.c_int64
        lib.lsr_alg2_reduce.restype = ctypes.c_int
        lib.lsr_alg2_reduce.argtypes = [vp, ctypes.c_int, i64, vp, vp, vp, vp, vp, ctypes.c_int, i64, i64, ctypes.c_int, vp]
        _lib = lib
    return _lib


class Alg2Forward:
    """Holds what Alg. 2 needs besides the inputs: the packing of the valid tokens (done once per batch,
    inside the timed call) and one tile of logits (M x tile_cols, reused for every tile)."""

    def __init__(self, H, W, bias, mask, tile_cols: int, logits_dtype=torch.float32):
        load_library()
        self.H, self.W, self.bias = H, W, bias
        self.B, self.S, self.D = H.shape
        self.V = W.shape[0]
        if tile_cols % 2 or self.V % 2:
            raise ValueError("the reduce kernel reads column pairs: tile_cols and |V| must be even")
        self.tile_cols = tile_cols
        self.logits_dtype = logits_dtype
        self.mask = mask
        dev = H.device
        self.Y = torch.empty((self.B, self.V), dtype=torch.float32, device=dev)
        self.I = torch.empty((self.B, self.V), dtype=torch.int32, device=dev)
        M_max = self.B * self.S
        self.logits = torch.empty((M_max, tile_cols), dtype=logits_dtype, device=dev)
        self.M = None
        self._mm_out = True

    def forward(self):
        # pack the valid tokens (Alg. 2 multiplies by the mask instead; packing is the cheaper reading)
        valid = self.mask.view(-1) != 0
        rows = torch.nonzero(valid).view(-1)
        lens = self.mask.view(self.B, self.S).ne(0).sum(dim=1)
        seq_row0 = torch.zeros(self.B + 1, dtype=torch.int32, device=self.H.device)
        seq_row0[1:] = lens.cumsum(0)
        row_pos = (rows % self.S).to(torch.int32)
        Hp = self.H.view(self.B * self.S, self.D).index_select(0, rows)
        M = Hp.shape[0]
        self.M = M
        stream = torch.cuda.current_stream().cuda_stream
        lib = _lib
        for v0 in range(0, self.V, self.tile_cols):
            C = min(self.tile_cols, self.V - v0)
            out = self.logits[:M, :C] if C == self.tile_cols else self.logits.view(-1)[: M * C].view(M, C)
            Wt = self.W[v0:v0 + C].t()
            if self.logits_dtype != torch.float32:
                torch.mm(Hp, Wt, out=out)
            elif self._mm_out:
                try:
                    torch.mm(Hp, Wt, out_dtype=torch.float32, out=out)
                except (TypeError, RuntimeError):
                    self._mm_out = False       # this torch build has no out= form of the widening mm
            if self.logits_dtype == torch.float32 and not self._mm_out:
                out = torch.mm(Hp, Wt, out_dtype=torch.float32)
            rc = lib.lsr_alg2_reduce(out.data_ptr(), 0 if self.logits_dtype == torch.float32 else 1, out.stride(0),
                                     seq_row0.data_ptr(), row_pos.data_ptr(), self.bias.data_ptr(),
                                     self.Y.data_ptr(), self.I.data_ptr(), self.B, self.V, v0, C, stream)
            if rc != 0:
                raise RuntimeError(f"lsr_alg2_reduce returned {rc}")
        return self.Y, self.I

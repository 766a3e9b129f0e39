"""Seeded synthetic workloads for the LSR LM head (inputs only; no head arithmetic).

The paper evaluates on hidden states of BERT-base / XLM-R-base sized encoders
(Experiments, Table 1, Fig. 2, Table 2).  Those activations and weights are not
available here, so every workload is random data of the same shape, value scale and
padding structure.  This module serves both the CPU oracle's tests and the GPU path,
so it contains nothing of the method itself: only random draws, a length-to-mask
expansion and the float32 -> bfloat16 storage rounding of the inputs.

Draw order per workload (one numpy Generator, seed = BASE_SEED + index):
H, W, bias, lengths, dY, Bernoulli keep-mask for dY (when the workload has one).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

BASE_SEED = 20260325


@dataclass(frozen=True)
class Workload:
    name: str
    index: int            # position in the benchmark's config list (seed offset)
    B: int
    S: int
    D: int
    V: int
    dtype: str            # "f32" or "bf16": storage type of H and W
    h_std: float
    w_std: float
    b_std: float
    len_lo: int
    len_hi: int
    backward: bool
    dy_keep: Optional[float]   # Bernoulli keep-probability applied to dY, or None (dense)
    what: str


WORKLOADS = {
    "c1_tiny_f32": Workload("c1_tiny_f32", 0, 2, 16, 64, 1000, "f32", 1.0, 0.05, 0.1, 1, 16, True, None,
                            "tiny fp32 head, CPU-checkable"),
    "c2_doc_fwd": Workload("c2_doc_fwd", 1, 32, 256, 768, 30522, "bf16", 1.0, 0.02, 0.02, 64, 256, False, None,
                           "BERT-base sized document encoding, forward only"),
    "c3_query_fwdbwd": Workload("c3_query_fwdbwd", 2, 256, 32, 768, 30522, "bf16", 1.0, 0.02, 0.02, 4, 32, True, 0.05,
                                "BERT-base sized query encoding, forward+backward, sparse dY"),
    "c4_xlmr_fwdbwd": Workload("c4_xlmr_fwdbwd", 3, 16, 256, 768, 250002, "bf16", 1.0, 0.02, 0.02, 32, 256, True, None,
                               "XLM-R-base sized head, forward+backward"),
    "c5_large_fwdbwd": Workload("c5_large_fwdbwd", 4, 64, 512, 1024, 250002, "bf16", 1.0, 0.02, 0.02, 128, 512, True, None,
                                "large multilingual training step, forward+backward"),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 storage (round-to-nearest-even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounding = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rounding) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class HeadInputs:
    """One batch.  H and W are float32 arrays holding exactly the stored values
    (already bf16-representable when dtype == "bf16"); H_bits / W_bits carry the
    bfloat16 storage for the device in that case."""
    workload: Workload
    H: np.ndarray                 # [B,S,D] float32
    W: np.ndarray                 # [V,D]   float32
    bias: np.ndarray              # [V]     float32
    lengths: np.ndarray           # [B]     int64
    mask: np.ndarray              # [B,S]   uint8, 1 = valid token
    dY: Optional[np.ndarray]      # [B,V]   float32 upstream gradient, or None
    H_bits: Optional[np.ndarray] = None   # uint16
    W_bits: Optional[np.ndarray] = None   # uint16

    @property
    def sum_len(self) -> int:
        return int(self.mask.sum())


def lengths_to_mask(lengths: np.ndarray, S: int) -> np.ndarray:
    """mask[b,s] = 1 for s < lengths[b] (padding at the end of each row)."""
    return (np.arange(S)[None, :] < np.asarray(lengths)[:, None]).astype(np.uint8)


def make_inputs(w: Workload, *, seed: Optional[int] = None, with_dy: Optional[bool] = None) -> HeadInputs:
    rng = np.random.default_rng(BASE_SEED + w.index if seed is None else seed)
    H = rng.standard_normal((w.B, w.S, w.D), dtype=np.float32) * np.float32(w.h_std)
    W = rng.standard_normal((w.V, w.D), dtype=np.float32) * np.float32(w.w_std)
    bias = rng.standard_normal(w.V, dtype=np.float32) * np.float32(w.b_std)
    lengths = rng.integers(w.len_lo, w.len_hi + 1, size=w.B)
    mask = lengths_to_mask(lengths, w.S)
    want_dy = w.backward if with_dy is None else with_dy
    dY = None
    if want_dy:
        dY = rng.standard_normal((w.B, w.V), dtype=np.float32)
        if w.dy_keep is not None:
            dY *= (rng.random((w.B, w.V), dtype=np.float32) < np.float32(w.dy_keep)).astype(np.float32)
    H_bits = W_bits = None
    if w.dtype == "bf16":
        H_bits = f32_to_bf16_bits(H)
        W_bits = f32_to_bf16_bits(W)
        H = bf16_bits_to_f32(H_bits)
        W = bf16_bits_to_f32(W_bits)
    return HeadInputs(w, H, W, bias, lengths, mask, dY, H_bits, W_bits)


def make_custom(B: int, S: int, D: int, V: int, *, dtype: str = "bf16", seed: int = 0,
                len_lo: int = 1, len_hi: Optional[int] = None, backward: bool = True,
                dy_keep: Optional[float] = None, w_std: float = 0.02, b_std: float = 0.02,
                h_std: float = 1.0, name: str = "custom") -> HeadInputs:
    """A workload of arbitrary shape with the same recipe (edge-case and sweep shapes)."""
    w = Workload(name, 0, B, S, D, V, dtype, h_std, w_std, b_std, len_lo,
                 S if len_hi is None else len_hi, backward, dy_keep, "custom shape")
    return make_inputs(w, seed=BASE_SEED + 1000 + seed)


def scattered_mask(rng: np.random.Generator, B: int, S: int, keep: float = 0.5) -> np.ndarray:
    """An arbitrary (non-suffix) attention mask; some rows may end up empty."""
    return (rng.random((B, S)) < keep).astype(np.uint8)

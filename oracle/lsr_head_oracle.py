"""Plain float64 CPU oracle of the sparse-lexical LM head (test infrastructure, not product).

What it computes, with the passage each function follows:

* ``forward``            Eq. 1 evaluated in the six-step order of Alg. 1 (standard LM head):
                         logits, +bias, activation log(1+ReLU(.)), mask, max over the sequence.
                         The whole B x S x C logit block is materialised per vocabulary chunk.
* ``forward_max_first``  the monotonicity reordering of Sec. 3 "Forward Pass": maximum of the raw
                         valid logits first, activation once afterwards.
* ``backward``           the gradient of Sec. 3 "Backward Pass" / Alg. 3: gate through the
                         derivative of log(1+ReLU(x)), route to the arg-max position.

Readings taken where the paper is silent or inconsistent:
  - the attention mask EXCLUDES positions from the arg-max (Eq. 1 multiplies after the
    activation, Alg. 1/2 before; all give the same Y, and exclusion keeps I on a valid token);
  - ties in the arg-max go to the lowest sequence index;
  - a row with no valid token yields Y = 0, I = 0 and no gradient;
  - the gate is strict: a maximum logit <= 0 passes no gradient;
  - the bias gradient (not listed among Alg. 3's outputs) is db[v] = sum_b g[b,v];
  - log is the natural logarithm.
The derivative is written here as 1/(1+x) from the oracle's own raw maximum x; the formula
printed in Alg. 3, delta*exp(-s_max) with s_max the saved output, is the same quantity written
another way and is what the device code uses, so agreement between them is a real check.

Pins (tests/test_oracle_*.py, no GPU): scalar brute force (oracle/brute_force.py), a hand-worked
example (tests/golden/), closed forms (W = 0, S = 1 linear layer, one-hot H), the exact
identity between both operator orders, invariants, central finite differences, and an
independent float64 autograd evaluation of the literal six-step formula.
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np

F64 = np.float64


def _as64(*arrays):
    return [np.asarray(a, dtype=F64) for a in arrays]


def logits_block(H: np.ndarray, W_rows: np.ndarray, bias_rows: np.ndarray) -> np.ndarray:
    """Alg. 1 steps 1-2: L[b,s,c] = sum_d H[b,s,d] * W_rows[c,d] + bias_rows[c]  (float64)."""
    H, W_rows, bias_rows = _as64(H, W_rows, bias_rows)
    B, S, D = H.shape
    L = H.reshape(B * S, D) @ W_rows.T
    L = L + bias_rows[None, :]
    return L.reshape(B, S, -1)


def forward(H, W, bias, mask, v_chunk: int = 4096) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Eq. 1 in Alg. 1's order.  Returns (Y[B,V] f64, I[B,V] int64, X[B,V] f64).

    X is the maximum raw (biased) logit over valid positions, -inf for a row without any.
    I is the lowest valid s attaining X, 0 for a row without valid positions.
    """
    H64, W64, b64 = _as64(H, W, bias)
    M = np.asarray(mask) != 0                       # [B,S]
    B, S, _ = H64.shape
    V = W64.shape[0]
    Y = np.empty((B, V), F64)
    X = np.empty((B, V), F64)
    I = np.empty((B, V), np.int64)
    Mf = M.astype(F64)[:, :, None]
    for v0 in range(0, V, v_chunk):
        v1 = min(V, v0 + v_chunk)
        L = logits_block(H64, W64[v0:v1], b64[v0:v1])        # steps 1-2, materialised
        A = np.log1p(np.maximum(L, 0.0))                      # steps 4-5 (Eq. 1: activation ...)
        A = A * Mf                                            # step 3   (... then the mask)
        Y[:, v0:v1] = A.max(axis=1)                           # step 6
        Lx = np.where(M[:, :, None], L, -np.inf)              # exclusion reading for the index
        X[:, v0:v1] = Lx.max(axis=1)
        I[:, v0:v1] = np.argmax(Lx, axis=1)                   # first occurrence = lowest s
    empty = ~M.any(axis=1)
    I[empty, :] = 0
    return Y, I, X


def forward_max_first(H, W, bias, mask, v_chunk: int = 4096) -> np.ndarray:
    """Sec. 3 reordering: Y = f(max over valid s of the raw logit), f(x) = log(1+ReLU(x))."""
    H64, W64, b64 = _as64(H, W, bias)
    M = np.asarray(mask) != 0
    B = H64.shape[0]
    V = W64.shape[0]
    Y = np.zeros((B, V), F64)
    for v0 in range(0, V, v_chunk):
        v1 = min(V, v0 + v_chunk)
        L = logits_block(H64, W64[v0:v1], b64[v0:v1])
        for b in range(B):
            if M[b].any():
                x = L[b][M[b]].max(axis=0)
                Y[b, v0:v1] = np.log1p(np.maximum(x, 0.0))
    return Y


def gate(dY, X) -> np.ndarray:
    """Alg. 3's gate: g = dY * f'(x) with f'(x) = 1/(1+x) for x > 0 and 0 otherwise."""
    dY64, X64 = _as64(dY, X)
    pos = X64 > 0.0
    g = np.zeros_like(dY64)
    g[pos] = dY64[pos] / (1.0 + X64[pos])
    return g


def backward_from_gate(H, W, g, I, v_chunk: int = 8192):
    """Alg. 3 routing given the gated gradient g[B,V] and indices I[B,V]:
    db[v] = sum_b g;  dW[v,:] = sum_b g[b,v] H[b,I[b,v],:];  dH[b,s,:] = sum_{v:I[b,v]=s} g[b,v] W[v,:]."""
    H64, W64, g64 = _as64(H, W, g)
    I = np.asarray(I).astype(np.int64)
    B, S, D = H64.shape
    V = W64.shape[0]
    db = g64.sum(axis=0)
    dW = np.zeros((V, D), F64)
    dH = np.zeros((B, S, D), F64)
    for b in range(B):
        nz = np.flatnonzero(g64[b])                 # pairs with g = 0 contribute nothing
        for c0 in range(0, nz.size, v_chunk):
            vs = nz[c0:c0 + v_chunk]                # distinct rows, so the indexed += is exact
            dW[vs] += g64[b, vs, None] * H64[b][I[b, vs]]
        for s in np.unique(I[b][nz]):
            sel = I[b] == s
            dH[b, s] = g64[b, sel] @ W64[sel]
    return dH, dW, db


def backward(H, W, bias, mask, dY, I_override: Optional[np.ndarray] = None, v_chunk: int = 4096):
    """Full analytic gradient.  Returns (dH, dW, db, g, I_used).

    With I_override the gradient is routed through the given indices (used when a device
    result legitimately picked the other member of a near-tie); the gate always comes from
    the oracle's own maximum logit."""
    _, I, X = forward(H, W, bias, mask, v_chunk=v_chunk)
    g = gate(dY, X)
    I_used = I if I_override is None else np.asarray(I_override).astype(np.int64)
    dH, dW, db = backward_from_gate(H, W, g, I_used)
    return dH, dW, db, g, I_used


def top2_gap(H, W, bias, mask, v_chunk: int = 4096) -> np.ndarray:
    """Difference between the largest and second largest valid logit per (b,v); +inf when a row
    has fewer than two valid positions.  Used to decide whether an arg-max mismatch is a near-tie."""
    H64, W64, b64 = _as64(H, W, bias)
    M = np.asarray(mask) != 0
    B = H64.shape[0]
    V = W64.shape[0]
    gap = np.full((B, V), np.inf)
    for v0 in range(0, V, v_chunk):
        v1 = min(V, v0 + v_chunk)
        L = logits_block(H64, W64[v0:v1], b64[v0:v1])
        for b in range(B):
            n = int(M[b].sum())
            if n >= 2:
                Lb = L[b][M[b]]
                part = np.partition(Lb, n - 2, axis=0)
                gap[b, v0:v1] = part[n - 1] - part[n - 2]
    return gap


def logit_at(H, W, bias, b_idx, s_idx, v_idx) -> np.ndarray:
    """Raw biased logits at listed (b,s,v) triples, one dot product each."""
    H64, W64, b64 = _as64(H, W, bias)
    return np.einsum("nd,nd->n", H64[b_idx, s_idx], W64[v_idx]) + b64[v_idx]

"""Comparison rules between the HIP path and the fp64 oracle (used by the GPU tests and smoke()).

Tolerances are those of the benchmark spec: max-abs error <= 2e-2 and max-rel error <= 1e-2 on
outputs and gradients; the arg-max must match exactly except where the two largest valid logits
differ by less than 1e-3.  Relative error is taken over elements whose reference magnitude is at
least 1e-2 of the tensor's largest magnitude (it is undefined at the exact zeros of Y and dH).
Gradients are compared with the oracle evaluated at the device's (validated) indices, because a
legitimate near-tie flip moves a whole row of dH.
"""
import numpy as np

from oracle import lsr_head_oracle as orc

ABS_TOL = 2e-2
REL_TOL = 1e-2
TIE_GAP = 1e-3


def check_close(name, got, ref, abs_tol=ABS_TOL, rel_tol=REL_TOL):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, f"{name}: shape {got.shape} vs {ref.shape}"
    assert np.all(np.isfinite(got)), f"{name}: non-finite values in the device result"
    err = np.abs(got - ref)
    max_abs = float(err.max()) if err.size else 0.0
    scale = float(np.abs(ref).max()) if ref.size else 0.0
    sel = np.abs(ref) >= 1e-2 * scale if scale > 0 else np.zeros_like(ref, bool)
    max_rel = float((err[sel] / np.abs(ref[sel])).max()) if sel.any() else 0.0
    assert max_abs <= abs_tol, f"{name}: max-abs {max_abs:.3e} > {abs_tol}"
    assert max_rel <= rel_tol, f"{name}: max-rel {max_rel:.3e} > {rel_tol}"
    return max_abs, max_rel


def check_close_bf16(name, got, ref):
    """For gradients delivered in bfloat16: each element within one bf16 step of the oracle (half a step
    of rounding, and as much again where float32 noise moves a value across a rounding boundary),
    |got - ref| <= 2^-8 |ref| + 2e-5.  Tighter than the fp32 bound for small entries, and the only
    meaningful bound for large ones (a dW entry of 15 rounds by up to 0.03)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, f"{name}: shape {got.shape} vs {ref.shape}"
    assert np.all(np.isfinite(got)), f"{name}: non-finite values in the device result"
    excess = np.abs(got - ref) - (2.0 ** -8 * np.abs(ref) + 2e-5)
    worst = float(excess.max()) if excess.size else 0.0
    assert worst <= 0.0, f"{name}: {int((excess > 0).sum())} elements beyond one bf16 step, worst excess {worst:.3e}"
    return float(np.abs(got - ref).max()) if got.size else 0.0


def check_index(H, W, bias, mask, I_gpu, I_ref, X_ref):
    """Exact match, or a near-tie: the device's position is valid and its logit is within TIE_GAP
    of the maximum.  Returns the number of near-tie flips."""
    I_gpu = np.asarray(I_gpu).astype(np.int64)
    S = np.asarray(mask).shape[1]
    assert I_gpu.min() >= 0 and I_gpu.max() < S, "index outside [0,S)"
    diff = np.argwhere(I_gpu != I_ref)
    if diff.shape[0] == 0:
        return 0
    bi, vi = diff[:, 0], diff[:, 1]
    si = I_gpu[bi, vi]
    assert np.all(np.asarray(mask)[bi, si] != 0), "device picked a masked position"
    lg = orc.logit_at(H, W, bias, bi, si, vi)
    short = X_ref[bi, vi] - lg
    assert np.all(short < TIE_GAP), f"{diff.shape[0]} index mismatches, worst logit shortfall {short.max():.3e}"
    return int(diff.shape[0])


def compare_forward(inp, Y_gpu, I_gpu, mask=None, v_sel=None, b_sel=None, v_chunk=4096):
    """Full or sliced forward comparison; returns (Y_ref, I_ref, X_ref, stats)."""
    mask = inp.mask if mask is None else mask
    H, W, bias = inp.H, inp.W, inp.bias
    if b_sel is not None:
        H, mask, Y_gpu = H[b_sel], mask[b_sel], Y_gpu[b_sel]
        I_gpu = None if I_gpu is None else I_gpu[b_sel]
    if v_sel is not None:
        W, bias, Y_gpu = W[v_sel], bias[v_sel], Y_gpu[:, v_sel]
        I_gpu = None if I_gpu is None else I_gpu[:, v_sel]
    Y_ref, I_ref, X_ref = orc.forward(H, W, bias, mask, v_chunk=v_chunk)
    stats = {"Y": check_close("Y", Y_gpu, Y_ref)}
    if I_gpu is not None:
        stats["index_flips"] = check_index(H, W, bias, mask, I_gpu, I_ref, X_ref)
    return Y_ref, I_ref, X_ref, stats


def compare_backward(inp, I_gpu, dH_gpu, dW_gpu, db_gpu, mask=None, v_sel=None, b_sel=None, v_chunk=4096,
                     bf16_grads=False):
    """Oracle gradient routed through the device's indices.  With v_sel only dW/db rows of the
    sample are compared (they are separable per vocabulary row); with b_sel only dH of those
    sequences (separable per sequence)."""
    mask = inp.mask if mask is None else mask
    H, W, bias, dY = inp.H, inp.W, inp.bias, inp.dY
    stats = {}
    close = check_close_bf16 if bf16_grads else check_close     # dH and dW; db is always float32
    if v_sel is None and b_sel is None:
        dH, dW, db, _, _ = orc.backward(H, W, bias, mask, dY, I_override=I_gpu, v_chunk=v_chunk)
        stats["dH"] = close("dH", dH_gpu, dH)
        stats["dW"] = close("dW", dW_gpu, dW)
        stats["db"] = check_close("db", db_gpu, db)
        return stats
    if v_sel is not None:
        _, dW, db, _, _ = orc.backward(H, W[v_sel], bias[v_sel], mask, dY[:, v_sel], I_override=I_gpu[:, v_sel],
                                        v_chunk=v_chunk)
        stats["dW"] = close("dW[sample]", dW_gpu[v_sel], dW)
        stats["db"] = check_close("db[sample]", db_gpu[v_sel], db)
    if b_sel is not None:
        dH, _, _, _, _ = orc.backward(H[b_sel], W, bias, mask[b_sel], dY[b_sel], I_override=I_gpu[b_sel], v_chunk=v_chunk)
        stats["dH"] = close("dH[sample]", dH_gpu[b_sel], dH)
    return stats

"""Do the oracle's pins bite?  Each case plants one plausible mistake in a copy of the oracle's source
(a dropped term, a wrong sign, a wrong index, a loosened condition) and requires that the pin battery
rejects the copy.  The untouched source must pass the same battery.  Everything runs on the CPU."""
import json
import os
import types

import numpy as np
import pytest

from oracle import brute_force

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE_SRC = os.path.join(os.path.dirname(HERE), "oracle", "lsr_head_oracle.py")
GOLDEN = os.path.join(HERE, "golden", "hand_example.json")


def load_oracle(edit=None):
    src = open(ORACLE_SRC).read()
    if edit is not None:
        old, new = edit
        assert src.count(old) == 1, f"mutation anchor not unique or missing: {old!r}"
        src = src.replace(old, new)
    mod = types.ModuleType("oracle_under_test")
    exec(compile(src, ORACLE_SRC, "exec"), mod.__dict__)
    return mod


def _case(seed, B=3, S=5, D=4, V=9):
    rng = np.random.default_rng(seed)
    H = rng.standard_normal((B, S, D))
    W = rng.standard_normal((V, D)) * 0.5
    bias = rng.standard_normal(V) * 0.4
    mask = (rng.random((B, S)) < 0.6).astype(np.uint8)
    mask[0, 1] = 1
    mask[B - 1, :] = 0                     # one row without valid tokens
    dY = rng.standard_normal((B, V))
    return H, W, bias, mask, dY


def pin_battery(orc):
    """Hand-worked example, scalar brute force on random masked cases, forced ties, finite differences."""
    g = json.load(open(GOLDEN))
    for case in g["cases"]:
        Y, I, _ = orc.forward(g["H"], g["W"], g["bias"], case["mask"])
        np.testing.assert_allclose(Y, case["Y"], atol=1e-15)
        assert np.array_equal(I, np.array(case["I"]))
        dH, dW, db, gate, _ = orc.backward(g["H"], g["W"], g["bias"], case["mask"], case["dY"])
        np.testing.assert_allclose(gate, case["g"], atol=1e-15)
        np.testing.assert_allclose(db, case["db"], atol=1e-15)
        np.testing.assert_allclose(dW, case["dW"], atol=1e-15)
        np.testing.assert_allclose(dH, case["dH"], atol=1e-15)
    for seed in (0, 1, 2, 3):
        H, W, bias, mask, dY = _case(seed)
        Y, I, _ = orc.forward(H, W, bias, mask, v_chunk=4)
        Yb, Ib, _ = brute_force.forward(H.tolist(), W.tolist(), bias.tolist(), mask.tolist())
        np.testing.assert_allclose(Y, np.array(Yb), rtol=1e-12, atol=1e-13)
        assert np.array_equal(I, np.array(Ib))
        np.testing.assert_allclose(orc.forward_max_first(H, W, bias, mask), np.array(Yb), rtol=1e-12, atol=1e-13)
        dH, dW, db, _, _ = orc.backward(H, W, bias, mask, dY, v_chunk=4)
        dHb, dWb, dbb = brute_force.backward(H.tolist(), W.tolist(), bias.tolist(), mask.tolist(), dY.tolist())
        np.testing.assert_allclose(dH, np.array(dHb), rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(dW, np.array(dWb), rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(db, np.array(dbb), rtol=1e-12, atol=1e-13)
    # exact ties: twins of a row must lose to the lowest position
    H, W, bias, mask, _ = _case(5, B=1, S=6)
    mask[:] = 1
    H[0, 4] = H[0, 1]
    H[0, 5] = H[0, 1]
    _, I, _ = orc.forward(H, W, bias, mask)
    assert not np.any(I >= 4)
    # central differences of sum(dY * Y) with respect to the bias, away from kinks
    H, W, bias, mask, dY = _case(21, B=2, S=4, D=3, V=6)
    mask[:] = 1
    _, _, X = orc.forward(H, W, bias, mask)
    assert np.min(np.abs(X)) > 1e-3
    _, _, db, _, _ = orc.backward(H, W, bias, mask, dY)
    eps = 1e-6
    for v in range(bias.size):
        bp, bm = bias.copy(), bias.copy()
        bp[v] += eps
        bm[v] -= eps
        fd = ((dY * orc.forward(H, W, bp, mask)[0]).sum() - (dY * orc.forward(H, W, bm, mask)[0]).sum()) / (2 * eps)
        assert abs(fd - db[v]) < 1e-6


def test_unmodified_oracle_passes_the_battery():
    pin_battery(load_oracle())


MUTANTS = {
    "bias dropped from the logits": ("L = L + bias_rows[None, :]", "L = L + 0.0 * bias_rows[None, :]"),
    "sign of the weights flipped": ("@ W_rows.T", "@ (-W_rows).T"),
    "index ignores the mask": ("Lx = np.where(M[:, :, None], L, -np.inf)              # exclusion",
                               "Lx = np.where(M[:, :, None], L, L)              # exclusion"),
    "output ignores the mask": ("A = A * Mf ", "A = A * 1.0 "),
    "ReLU replaced by abs": ("A = np.log1p(np.maximum(L, 0.0))", "A = np.log1p(np.abs(L))"),
    "log1p argument halved": ("A = np.log1p(np.maximum(L, 0.0))", "A = np.log1p(0.5 * np.maximum(L, 0.0))"),
    "last position wins ties": ("I[:, v0:v1] = np.argmax(Lx, axis=1)",
                                "I[:, v0:v1] = Lx.shape[1] - 1 - np.argmax(Lx[:, ::-1], axis=1)"),
    "gate uses exp(-x) of the raw logit": ("g[pos] = dY64[pos] / (1.0 + X64[pos])", "g[pos] = dY64[pos] * np.exp(-X64[pos])"),
    "gate open below zero": ("pos = X64 > 0.0", "pos = X64 > -0.9"),
    "bias gradient drops a sequence": ("db = g64.sum(axis=0)", "db = g64[1:].sum(axis=0)"),
    "dW gathers the neighbouring position": ("H64[b][I[b, vs]]", "H64[b][np.minimum(I[b, vs] + 1, S - 1)]"),
    "dH sign flipped": ("dH[b, s] = g64[b, sel] @ W64[sel]", "dH[b, s] = -(g64[b, sel] @ W64[sel])"),
    "dH sums ungated rows too": ("sel = I[b] == s", "sel = (I[b] == s) | (np.arange(V) == 0)"),
    "max-first order forgets the activation": ("Y[b, v0:v1] = np.log1p(np.maximum(x, 0.0))", "Y[b, v0:v1] = np.maximum(x, 0.0)"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name):
    mutant = load_oracle(MUTANTS[name])
    with pytest.raises(AssertionError):
        pin_battery(mutant)

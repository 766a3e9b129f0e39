"""Pins for the oracle's analytic gradient (CPU only)."""
import json
import os

import numpy as np
import pytest
import torch

from oracle import brute_force
from oracle import lsr_head_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_example.json")


def _case(seed, B=3, S=5, D=4, V=9, empty_row=True):
    rng = np.random.default_rng(seed)
    H = rng.standard_normal((B, S, D))
    W = rng.standard_normal((V, D)) * 0.5
    bias = rng.standard_normal(V) * 0.2
    mask = (rng.random((B, S)) < 0.7).astype(np.uint8)
    mask[0, 1] = 1
    if empty_row:
        mask[B - 1, :] = 0
    dY = rng.standard_normal((B, V))
    return H, W, bias, mask, dY


def test_hand_worked_example_backward():
    g = json.load(open(GOLDEN))
    for case in g["cases"]:
        dH, dW, db, gate, _ = orc.backward(g["H"], g["W"], g["bias"], case["mask"], case["dY"])
        np.testing.assert_allclose(gate, case["g"], atol=1e-15)
        np.testing.assert_allclose(db, case["db"], atol=1e-15)
        np.testing.assert_allclose(dW, case["dW"], atol=1e-15)
        np.testing.assert_allclose(dH, case["dH"], atol=1e-15)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_matches_scalar_brute_force(seed):
    H, W, bias, mask, dY = _case(seed)
    dH, dW, db, _, _ = orc.backward(H, W, bias, mask, dY, v_chunk=4)
    dHb, dWb, dbb = brute_force.backward(H.tolist(), W.tolist(), bias.tolist(), mask.tolist(), dY.tolist())
    np.testing.assert_allclose(dH, np.array(dHb), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dW, np.array(dWb), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(db, np.array(dbb), rtol=1e-12, atol=1e-13)


def test_central_finite_differences():
    # loss = sum(dY * Y); away from kinks (|x| and the top-2 gap both far above the step)
    H, W, bias, mask, dY = _case(21, B=2, S=4, D=3, V=6, empty_row=False)
    _, _, X = orc.forward(H, W, bias, mask)
    gap = orc.top2_gap(H, W, bias, mask)
    assert np.min(np.abs(X)) > 1e-3 and np.min(gap) > 1e-3, "pick another seed: too close to a kink"
    dH, dW, db, _, _ = orc.backward(H, W, bias, mask, dY)

    def loss(H_, W_, b_):
        return float((dY * orc.forward(H_, W_, b_, mask)[0]).sum())

    eps = 1e-6
    for arr, grad, which in ((H, dH, 0), (W, dW, 1), (bias, db, 2)):
        num = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            args_p = [H.copy(), W.copy(), bias.copy()]
            args_m = [H.copy(), W.copy(), bias.copy()]
            args_p[which][idx] += eps
            args_m[which][idx] -= eps
            num[idx] = (loss(*args_p) - loss(*args_m)) / (2 * eps)
        np.testing.assert_allclose(grad, num, rtol=1e-6, atol=1e-8)


def test_autograd_of_the_literal_six_step_head():
    # Independent route: float64 autograd through Alg. 1's operator sequence (library routine).
    H, W, bias, mask, dY = _case(33, B=3, S=6, D=5, V=12)
    tH = torch.tensor(H, dtype=torch.float64, requires_grad=True)
    tW = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    tb = torch.tensor(bias, dtype=torch.float64, requires_grad=True)
    tM = torch.tensor(mask, dtype=torch.float64)
    L = tH @ tW.T
    L = L + tb
    A = torch.log1p(torch.relu(L)) * tM[:, :, None]
    Y = A.max(dim=1).values
    Y.backward(torch.tensor(dY, dtype=torch.float64))
    dH, dW, db, _, _ = orc.backward(H, W, bias, mask, dY)
    # (random data: no exact ties, so the sub-gradient choice of max() does not matter)
    np.testing.assert_allclose(dH, tH.grad.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dW, tW.grad.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(db, tb.grad.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(orc.forward(H, W, bias, mask)[0], Y.detach().numpy(), rtol=1e-14, atol=1e-15)


def test_single_position_reduces_to_linear_layer_backward():
    rng = np.random.default_rng(4)
    B, D, V = 4, 5, 7
    H = rng.standard_normal((B, 1, D))
    W = rng.standard_normal((V, D)) * 0.5
    bias = rng.standard_normal(V) * 0.1
    dY = rng.standard_normal((B, V))
    dH, dW, db, g, _ = orc.backward(H, W, bias, np.ones((B, 1), np.uint8), dY)
    lin = H[:, 0] @ W.T + bias
    g_ref = np.where(lin > 0, dY / (1 + lin), 0.0)
    np.testing.assert_allclose(g, g_ref, atol=1e-15)
    np.testing.assert_allclose(dW, g_ref.T @ H[:, 0], atol=1e-13)
    np.testing.assert_allclose(dH[:, 0], g_ref @ W, atol=1e-13)
    np.testing.assert_allclose(db, g_ref.sum(0), atol=1e-14)


def test_gradient_invariants():
    H, W, bias, mask, dY = _case(55, B=4, S=7, D=6, V=40)
    Y, I, X = orc.forward(H, W, bias, mask)
    dH, dW, db, g, _ = orc.backward(H, W, bias, mask, dY)
    # the saved output gives the same gate: exp(-Y) == 1/(1+x) on x > 0  (Alg. 3 as printed)
    np.testing.assert_allclose(g, np.where(Y > 0, dY * np.exp(-Y), 0.0), rtol=1e-13, atol=1e-15)
    # no gradient from a row without valid tokens; none to masked or unselected positions
    assert np.all(g[-1] == 0) and np.all(dH[-1] == 0)
    for b in range(4):
        used = set(I[b][g[b] != 0].tolist())
        for s in range(7):
            if s not in used:
                assert np.all(dH[b, s] == 0)
            if mask[b, s] == 0:
                assert np.all(dH[b, s] == 0)
    # sum over positions is a dense product; inner-product identities
    np.testing.assert_allclose(dH.sum(axis=1), g @ W, atol=1e-12)
    safeX = np.where(np.isfinite(X), X, 0.0)
    total = float((g * (safeX - bias[None, :])).sum())
    np.testing.assert_allclose((dH * H).sum(), total, rtol=1e-12)
    np.testing.assert_allclose((dW * W).sum(), total, rtol=1e-12)
    np.testing.assert_allclose(db, g.sum(0), atol=1e-14)


def test_strict_gate_at_the_kink():
    # a maximum logit of exactly 0 passes no gradient (ReLU'(0) = 0)
    H = np.array([[[1.0, 0.0]]])
    W = np.array([[0.0, 1.0], [2.0, 0.0]])
    bias = np.array([0.0, 0.0])
    dH, dW, db, g, _ = orc.backward(H, W, bias, np.ones((1, 1), np.uint8), np.ones((1, 2)))
    assert g[0, 0] == 0.0 and g[0, 1] == pytest.approx(1.0 / 3.0)
    assert db[0] == 0.0 and np.all(dW[0] == 0.0)


def test_index_override_routes_but_keeps_the_gate():
    H, W, bias, mask, dY = _case(77, B=2, S=4, D=3, V=5, empty_row=False)
    mask[:] = 1
    _, I, _ = orc.forward(H, W, bias, mask)
    I2 = (I + 1) % 4
    dH, dW, db, g, used = orc.backward(H, W, bias, mask, dY, I_override=I2)
    assert np.array_equal(used, I2)
    np.testing.assert_allclose(db, g.sum(0))
    for v in range(5):
        np.testing.assert_allclose(dW[v], sum(g[b, v] * H[b, I2[b, v]] for b in range(2)), atol=1e-14)

"""Pins for the oracle's forward (CPU only).  Each test checks the oracle against something
the paper or the mathematics fixes, not against itself."""
import json
import math
import os

import numpy as np
import pytest

from oracle import brute_force
from oracle import lsr_head_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_example.json")


def _rand(rng, B, S, D, V, w_std=0.3):
    H = rng.standard_normal((B, S, D))
    W = rng.standard_normal((V, D)) * w_std
    bias = rng.standard_normal(V) * 0.2
    return H, W, bias


def test_hand_worked_example_forward():
    g = json.load(open(GOLDEN))
    for case in g["cases"]:
        Y, I, _ = orc.forward(g["H"], g["W"], g["bias"], case["mask"])
        np.testing.assert_allclose(Y, case["Y"], rtol=0, atol=1e-15)
        assert I.tolist() == case["I"]
    # the stored decimals are the logs named next to them
    assert g["cases"][0]["Y"][0] == [math.log(3.0), math.log(2.5)]
    assert g["cases"][1]["Y"][0] == [math.log(2.0), 0.0]


@pytest.mark.parametrize("seed,B,S,D,V,maskmode", [
    (0, 2, 5, 3, 7, "suffix"), (1, 3, 4, 2, 5, "scatter"), (2, 1, 1, 4, 6, "full"),
    (3, 3, 6, 3, 4, "with_empty_row"),
])
def test_matches_scalar_brute_force(seed, B, S, D, V, maskmode):
    rng = np.random.default_rng(seed)
    H, W, bias = _rand(rng, B, S, D, V)
    if maskmode == "suffix":
        mask = (np.arange(S)[None] < rng.integers(1, S + 1, B)[:, None]).astype(np.uint8)
    elif maskmode == "scatter":
        mask = (rng.random((B, S)) < 0.6).astype(np.uint8)
        mask[0, 2] = 1
    elif maskmode == "full":
        mask = np.ones((B, S), np.uint8)
    else:
        mask = (rng.random((B, S)) < 0.7).astype(np.uint8)
        mask[1, :] = 0
    Y, I, X = orc.forward(H, W, bias, mask, v_chunk=3)
    Yb, Ib, Xb = brute_force.forward(H.tolist(), W.tolist(), bias.tolist(), mask.tolist())
    np.testing.assert_allclose(Y, np.array(Yb), rtol=1e-13, atol=1e-13)
    assert I.tolist() == Ib
    np.testing.assert_allclose(X, np.array(Xb), rtol=1e-13, atol=1e-13)


def test_operator_orders_agree_exactly():
    # Sec. 3: f monotone => max_s f(l) == f(max_s l); in float64 this is exact, not approximate.
    rng = np.random.default_rng(11)
    H, W, bias = _rand(rng, 4, 9, 8, 50)
    mask = (rng.random((4, 9)) < 0.7).astype(np.uint8)
    mask[2, :] = 0
    # (same vocabulary chunking on both sides so the library matmul rounds the logits identically)
    Y, _, _ = orc.forward(H, W, bias, mask, v_chunk=16)
    Y2 = orc.forward_max_first(H, W, bias, mask, v_chunk=16)
    assert np.array_equal(Y, Y2)
    Y3 = orc.forward_max_first(H, W, bias, mask, v_chunk=7)
    np.testing.assert_allclose(Y, Y3, rtol=1e-14, atol=1e-15)


def test_closed_form_zero_weights():
    rng = np.random.default_rng(5)
    H, _, bias = _rand(rng, 3, 4, 5, 9)
    mask = np.array([[1, 1, 0, 0], [0, 0, 0, 0], [0, 1, 0, 1]], np.uint8)
    Y, I, _ = orc.forward(H, np.zeros((9, 5)), bias, mask)
    expect = np.log1p(np.maximum(bias, 0.0))
    np.testing.assert_allclose(Y[0], expect, atol=1e-15)
    np.testing.assert_allclose(Y[2], expect, atol=1e-15)
    assert np.all(Y[1] == 0.0)
    # all valid logits tie at bias[v]: the lowest valid index wins
    assert np.all(I[0] == 0) and np.all(I[2] == 1) and np.all(I[1] == 0)


def test_closed_form_single_position_is_linear_layer():
    rng = np.random.default_rng(6)
    H, W, bias = _rand(rng, 5, 1, 6, 11)
    Y, I, X = orc.forward(H, W, bias, np.ones((5, 1), np.uint8))
    lin = H[:, 0, :] @ W.T + bias
    np.testing.assert_allclose(X, lin, rtol=1e-14, atol=1e-14)
    np.testing.assert_allclose(Y, np.log1p(np.maximum(lin, 0.0)), rtol=1e-14, atol=1e-14)
    assert np.all(I == 0)


def test_closed_form_one_hot_hidden_states():
    # H[b,s,:] = e_{k_s}  =>  logit[b,s,v] = W[v,k_s] + bias[v]
    rng = np.random.default_rng(7)
    D, V, S = 6, 8, 4
    W = rng.standard_normal((V, D))
    bias = rng.standard_normal(V) * 0.1
    ks = np.array([3, 0, 5, 3])
    H = np.zeros((1, S, D))
    H[0, np.arange(S), ks] = 1.0
    mask = np.array([[1, 1, 1, 0]], np.uint8)
    Y, I, _ = orc.forward(H, W, bias, mask)
    cols = W[:, ks[:3]]                               # [V,3]
    np.testing.assert_allclose(Y[0], np.log1p(np.maximum(cols.max(axis=1) + bias, 0.0)), atol=1e-15)
    assert np.array_equal(I[0], cols.argmax(axis=1))


def test_invariants_nonnegative_masked_rows_and_masked_positions():
    rng = np.random.default_rng(8)
    H, W, bias = _rand(rng, 4, 7, 5, 30)
    mask = (rng.random((4, 7)) < 0.6).astype(np.uint8)
    mask[3, :] = 0
    mask[0, 0] = 1
    Y, I, _ = orc.forward(H, W, bias, mask)
    assert np.all(Y >= 0.0)
    assert np.all(Y[3] == 0.0) and np.all(I[3] == 0)
    # the index always names a valid position where one exists
    for b in range(3):
        if mask[b].any():
            assert np.all(mask[b][I[b]] == 1)
    # hidden states at masked positions are irrelevant
    H2 = H.copy()
    H2[mask == 0] = rng.standard_normal((int((mask == 0).sum()), 5)) * 100.0
    Y2, I2, _ = orc.forward(H2, W, bias, mask)
    assert np.array_equal(Y, Y2) and np.array_equal(I, I2)


def test_invariant_permuting_valid_positions():
    rng = np.random.default_rng(9)
    H, W, bias = _rand(rng, 2, 6, 4, 20)
    mask = np.array([[1, 1, 1, 1, 0, 0], [1, 1, 1, 1, 1, 1]], np.uint8)
    Y, I, _ = orc.forward(H, W, bias, mask)
    perm = np.array([2, 0, 3, 1, 4, 5])                # permutes the 4 valid slots of row 0
    Hp = H.copy()
    Hp[0] = H[0][perm]                                 # new position j holds old position perm[j]
    Yp, Ip, _ = orc.forward(Hp, W, bias, mask)
    np.testing.assert_allclose(Yp, Y, rtol=0, atol=1e-15)
    assert np.array_equal(perm[Ip[0]], I[0])           # the index follows the token
    assert np.array_equal(Ip[1], I[1])


def test_forced_ties_pick_lowest_index():
    rng = np.random.default_rng(10)
    H, W, bias = _rand(rng, 1, 5, 4, 12)
    H[0, 3] = H[0, 1]                                  # identical rows => exactly equal logits
    H[0, 4] = H[0, 1]
    Y, I, _ = orc.forward(H, W, bias, np.ones((1, 5), np.uint8))
    assert not np.any(I == 3) and not np.any(I == 4)
    assert np.any(I == 1)
    mask = np.array([[1, 0, 1, 1, 1]], np.uint8)       # now position 1 is excluded: 3 is the lowest twin
    _, I2, _ = orc.forward(H, W, bias, mask)
    assert not np.any(I2 == 1) and not np.any(I2 == 4)


def test_memory_arithmetic_of_the_paper():
    # Sec. 1 / Sec. 3: B = S = 512, |V| = 30522 in half precision: logits 16 GB, reduced output ~31 MB
    B = S = 512
    V = 30522
    assert round(B * S * V * 2 / 1e9) == 16
    assert round(B * V * 2 / 1e6) == 31


def test_top2_gap_and_logit_at():
    rng = np.random.default_rng(12)
    H, W, bias = _rand(rng, 2, 5, 3, 6)
    mask = np.array([[1, 1, 1, 0, 0], [1, 0, 0, 0, 0]], np.uint8)
    gap = orc.top2_gap(H, W, bias, mask)
    L = orc.logits_block(H, W, bias)
    srt = np.sort(L[0, :3], axis=0)
    np.testing.assert_allclose(gap[0], srt[-1] - srt[-2], atol=1e-14)
    assert np.all(np.isinf(gap[1]))
    got = orc.logit_at(H, W, bias, np.array([0, 1]), np.array([2, 0]), np.array([4, 5]))
    np.testing.assert_allclose(got, [L[0, 2, 4], L[1, 0, 5]], atol=1e-14)

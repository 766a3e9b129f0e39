"""Parity at the benchmark's full sizes (|V| = 250002), in the launch configuration bench.py times.
The oracle cannot materialise these logits in seconds, so it is evaluated on what separates
exactly: a stratified sample of vocabulary rows for all sequences (Y, I, dW, db are independent per
vocabulary row) and whole sampled sequences over the full vocabulary (Y, I, dH are independent per
sequence).  Properties that hold at any size cover the rest."""
import numpy as np
import pytest
import torch

from paper_2603_25011_amd import inputs as wl
from paper_2603_25011_amd.harness import DeviceHead
from tests import parity

pytestmark = pytest.mark.gpu


def vocab_sample(V, n_random_tiles, rng, tile=256):
    n_tiles = (V + tile - 1) // tile
    tiles = {0, 1, n_tiles - 2, n_tiles - 1} | set(rng.choice(n_tiles, n_random_tiles, replace=False).tolist())
    rows = np.concatenate([np.arange(t * tile, min(V, (t + 1) * tile)) for t in sorted(tiles)])
    return rows


def fullsize_case(name, n_tiles, b_sel):
    w = wl.WORKLOADS[name]
    inp = wl.make_inputs(w)
    head = DeviceHead(inp)
    head.poison_outputs()
    head.forward()
    head.backward()
    torch.cuda.synchronize()
    Y, I = head.Y.cpu().numpy(), head.I.cpu().numpy()
    dH, dW, db = head.dH.cpu().numpy(), head.dW.cpu().numpy(), head.db.cpu().numpy()
    del head
    torch.cuda.empty_cache()
    # properties at full size
    assert np.all(np.isfinite(Y)) and np.all(Y >= 0)
    assert I.min() >= 0 and np.all(I < inp.lengths[:, None]), "index must name a valid (unpadded) token"
    assert np.all(np.isfinite(dH)) and np.all(np.isfinite(dW)) and np.all(np.isfinite(db))
    assert np.all(dH[inp.mask == 0] == 0.0)
    g = np.where(Y > 0, inp.dY.astype(np.float64) * np.exp(-Y.astype(np.float64)), 0.0)
    np.testing.assert_allclose(db, g.sum(0), rtol=1e-4, atol=1e-4)
    # sum_s dH[b,s,:] = sum_v g[b,v] W[v,:]  (dense product, independent of the routing)
    b0 = b_sel[0]
    np.testing.assert_allclose(dH[b0].sum(0), g[b0] @ inp.W.astype(np.float64), rtol=2e-3, atol=2e-3)
    # sampled vocabulary rows, all sequences
    rng = np.random.default_rng(1)
    vs = vocab_sample(w.V, n_tiles, rng)
    stats = parity.compare_forward(inp, Y, I, v_sel=vs)[3]
    stats.update(parity.compare_backward(inp, I, dH, dW, db, v_sel=vs))
    # sampled sequences, whole vocabulary
    bs = np.array(b_sel)
    stats["seq"] = parity.compare_forward(inp, Y, I, b_sel=bs)[3]
    stats.update(parity.compare_backward(inp, I, dH, dW, db, b_sel=bs))
    print(name, "rows sampled:", vs.size, stats)


def test_c4_xlmr_sized_head():
    fullsize_case("c4_xlmr_fwdbwd", n_tiles=28, b_sel=[0, 15])


def test_c5_large_training_step():
    fullsize_case("c5_large_fwdbwd", n_tiles=60, b_sel=[63])

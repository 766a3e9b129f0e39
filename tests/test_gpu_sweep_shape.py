"""Parity at one shape of the paper's head-only sweeps (Sec. 4: sequence-length sweep at B=128,
|V|=30522; Table 2's longest row, S=8192), on sampled outputs: three vocabulary tiles for all
sequences and one whole sequence over the full vocabulary.  At this shape a sequence spans 32 tiles of
the packed forward, the bucket sort places directly (S above 1024) and the dH gather serves eight
buckets per wave."""
import numpy as np
import pytest
import torch

from oracle import lsr_head_oracle as orc
from paper_2603_25011_amd import binding as lsr
from paper_2603_25011_amd import inputs as wl
from paper_2603_25011_amd.harness import DeviceHead
from tests import parity

pytestmark = pytest.mark.gpu


def test_long_sequence_sweep_shape_sampled():
    B, S, D, V = 128, 8192, 768, 30522
    plan = lsr.lsr_head_plan(B, S, D, V, lsr.LSR_BF16)
    assert plan["sort_places_through_lds"] == 0 and plan["dh_buckets_per_wave"] == 8
    inp = wl.make_custom(B, S, D, V, seed=8192, len_lo=4096, name="sweep_seq_8192")
    head = DeviceHead(inp)
    head.poison_outputs()
    head.forward()
    head.backward()
    torch.cuda.synchronize()
    Y, I = head.Y.cpu().numpy(), head.I.cpu().numpy()
    dH, dW, db = head.dH.cpu().numpy(), head.dW.cpu().numpy(), head.db.cpu().numpy()
    del head
    torch.cuda.empty_cache()
    assert np.all(np.isfinite(Y)) and np.all(Y >= 0)
    assert I.min() >= 0 and np.all(I < inp.lengths[:, None])
    assert np.all(np.isfinite(dW)) and np.all(np.isfinite(db))
    g = np.where(Y > 0, inp.dY.astype(np.float64) * np.exp(-Y.astype(np.float64)), 0.0)
    np.testing.assert_allclose(db, g.sum(0), rtol=1e-4, atol=1e-4)
    np.testing.assert_allclose(dH.sum(axis=1, dtype=np.float64), g @ inp.W.astype(np.float64), rtol=2e-3, atol=2e-3)
    print("device results checked for the size-independent properties", flush=True)
    # first, last (ragged) and one inner vocabulary tile, all sequences
    n_tiles = (V + 255) // 256
    vs = np.concatenate([np.arange(t * 256, min(V, (t + 1) * 256)) for t in (0, 57, n_tiles - 1)])
    _, _, X_ref, stats = parity.compare_forward(inp, Y, I, v_sel=vs, v_chunk=128)
    _, dW_ref, db_ref = orc.backward_from_gate(inp.H, inp.W[vs], orc.gate(inp.dY[:, vs], X_ref), I[:, vs])
    stats["dW"] = parity.check_close("dW[sample]", dW[vs], dW_ref)
    stats["db"] = parity.check_close("db[sample]", db[vs], db_ref)
    print("vocabulary rows sampled:", vs.size, stats, flush=True)
    # one whole sequence (not the first: its blocks start inside a tile)
    bs = np.array([77])
    _, _, X_ref, stats = parity.compare_forward(inp, Y, I, b_sel=bs, v_chunk=1024)
    dH_ref, _, _ = orc.backward_from_gate(inp.H[bs], inp.W, orc.gate(inp.dY[bs], X_ref), I[bs])
    stats["dH"] = parity.check_close("dH[sample]", dH[bs], dH_ref)
    assert np.all(dH[bs][inp.mask[bs] == 0] == 0.0)
    print("sequence 77, length", int(inp.lengths[77]), stats)

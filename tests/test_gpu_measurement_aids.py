"""The measurement aids bench.py quotes beside the head: the copy probe copies what it says it copies,
the probes return plausible rates, and the Alg. 2 comparator (Sec. 3, Alg. 2: a library GEMM per
vocabulary tile, then a reduce kernel) agrees with the oracle, so the time bench.py prints for it is
the time of a correct computation."""
import numpy as np
import pytest
import torch

from paper_2603_25011_amd import binding as lsr
from paper_2603_25011_amd import inputs as wl
from paper_2603_25011_amd.alg2_comparator import Alg2Forward
from paper_2603_25011_amd.harness import DeviceHead
from tests import parity

pytestmark = pytest.mark.gpu


def test_copy_probe_copies_and_reports_a_rate():
    n = 64 << 20
    g = torch.Generator(device="cuda:0").manual_seed(5)
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda:0", generator=g)
    dst = torch.zeros_like(src)
    rate = lsr.lsr_copy_probe(dst, src, n, launches=2)
    assert torch.equal(dst, src)
    assert 100.0 < rate < 16000.0, rate          # GB/s read + written; twice HBM's 8 TB/s bounds it
    with pytest.raises(lsr.LsrError):
        lsr.lsr_copy_probe(dst, src, n - 8, launches=2)      # not a multiple of 16


def test_gather_probe_rates_fall_with_the_window():
    table = torch.full((256 << 20,), 0x3C00, dtype=torch.int16, device="cuda:0")     # 512 MiB
    out = torch.empty(64 << 20, dtype=torch.uint8, device="cuda:0")
    small = lsr.lsr_gather_probe(table, 2 << 20, 512, out, launches=2)
    large = lsr.lsr_gather_probe(table, 512 << 20, 128, out, launches=2)
    assert small > large > 100.0, (small, large)
    with pytest.raises(lsr.LsrError):
        lsr.lsr_gather_probe(table, 2 << 20, 16, out[:1024], launches=1)             # out too small


@pytest.mark.parametrize("logits,tile_cols", [(torch.float32, 4096), (torch.float32, 1000), (torch.bfloat16, 4096)])
def test_alg2_comparator_matches_the_oracle(logits, tile_cols):
    inp = wl.make_custom(6, 96, 128, 9002, seed=77, len_lo=1, name="alg2_small")
    head = DeviceHead(inp)
    alg2 = Alg2Forward(head.H, head.W, head.bias, head.mask, tile_cols, logits)
    Y, I = alg2.forward()
    torch.cuda.synchronize()
    Y, I = Y.cpu().numpy(), I.cpu().numpy()
    assert I.min() >= 0 and np.all(I < inp.lengths[:, None])
    if logits == torch.float32:
        parity.compare_forward(inp, Y, I)
    else:
        # logits rounded to bf16 before the maximum: values within bf16 rounding of the oracle's, and the
        # index may name any token whose logit rounds to the same bf16 value (not the paper's arg-max rule)
        Y_ref, _, _ = parity.orc.forward(inp.H, inp.W, inp.bias, inp.mask)
        np.testing.assert_allclose(Y, Y_ref, rtol=2.0 ** -7, atol=2.0 ** -7)

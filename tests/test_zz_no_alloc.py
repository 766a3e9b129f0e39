"""lsr_head_forward_static (the forward that allocates nothing: its scratch is a static device array
inside the library) against lsr_head_forward on the same inputs, through the C ABI: two calls in a
row, the second on a smaller problem, so that whatever the first call left in the shared array is
there when the second runs.  Outputs must be identical (same kernels, same order of operations), and
the first pair is also held to the oracle."""
import numpy as np
import pytest
import torch

from paper_2603_25011_amd import binding as lsr
from paper_2603_25011_amd import inputs as wl
from paper_2603_25011_amd.harness import DeviceHead
from tests import parity

pytestmark = pytest.mark.gpu


def both_forwards(inp, want_index=True):
    head = DeviceHead(inp, want_index=want_index, want_backward=False)
    head.poison_outputs()
    head.forward()
    torch.cuda.synchronize()
    Y_ref = head.Y.clone()
    I_ref = head.I.clone() if want_index else None
    head.poison_outputs()
    before = torch.cuda.memory_allocated()
    lsr.lsr_head_forward_static(head.B, head.S, head.D, head.V, head.dt, head.H, head.W, head.bias, head.mask,
                                head.Y, head.I)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(head.Y, Y_ref)
    if want_index:
        assert torch.equal(head.I, I_ref)
    return head


def test_static_scratch_forward_matches_the_workspace_forward_twice_in_a_row():
    big = wl.make_custom(24, 300, 128, 3000, seed=71, len_lo=5, backward=False)
    small = wl.make_custom(3, 40, 64, 333, seed=72, len_lo=1, backward=False)
    head = both_forwards(big)
    print(parity.compare_forward(big, head.Y.cpu().numpy(), head.I.cpu().numpy())[3])
    head = both_forwards(small)
    print(parity.compare_forward(small, head.Y.cpu().numpy(), head.I.cpu().numpy())[3])
    # fp32 path and the index-free forward go through the same array
    both_forwards(wl.make_inputs(wl.WORKLOADS["c1_tiny_f32"], with_dy=False))
    both_forwards(wl.make_custom(5, 64, 128, 700, seed=73, backward=False), want_index=False)


def test_static_scratch_forward_rejects_shapes_beyond_its_array():
    # the forward scratch grows with B*S: 65535 sequences of 1024 positions need far more than the array holds
    need = lsr.lsr_head_workspace_bytes(4096, 1024, 64, 16, lsr.LSR_BF16, False)
    assert need > lsr.LSR_STATIC_SCRATCH_BYTES
    with pytest.raises(lsr.LsrError) as e:
        lsr.lsr_head_forward_static(4096, 1024, 64, 16, lsr.LSR_BF16, 4096, 4096, 4096, 4096, 4096, 4096, stream=0)
    assert e.value.status == 8

"""The forward and backward calls allocate nothing, never synchronise and take their stream from the
caller, so they can be recorded into a HIP graph.  The graph is replayed several times, with eager work
and synchronisations in between and with changed inputs, and every replay is compared with the eager
result on the same inputs."""
import pytest
import torch

from paper_2603_25011_amd import inputs as wl
from paper_2603_25011_amd.harness import DeviceHead

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("B,S,D,V", [
    (6, 70, 128, 900),        # small: the dW gather runs on the library's auxiliary stream beside dH
    (3, 40, 64, 70000),       # dH gathered in three vocabulary chunks (three launches in the graph)
])
def test_forward_backward_replayed_from_a_graph(B, S, D, V):
    inp = wl.make_custom(B, S, D, V, seed=B * 100 + S, len_lo=3)
    head = DeviceHead(inp)
    head.forward()                      # first calls create the library's per-device stream and events
    head.backward()
    torch.cuda.synchronize()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            head.forward()
            head.backward()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    for scale in (1.0, -0.5, 2.0):
        head.dY.copy_(torch.from_numpy(inp.dY).to(head.dev) * scale)
        head.bias.add_(0.01 * scale)
        # eager reference on the same inputs
        head.poison_outputs()
        head.forward()
        head.backward()
        torch.cuda.synchronize()
        ref = [t.clone() for t in (head.Y, head.I, head.dH, head.dW, head.db)]
        # unrelated eager work between the replays
        junk = torch.randn(1 << 20, device=head.dev)
        junk = (junk * 2).sum()
        head.poison_outputs()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip((head.Y, head.I, head.dH, head.dW, head.db), ref):
            assert torch.equal(got, want)

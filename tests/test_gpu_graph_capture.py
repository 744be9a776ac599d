"""The whole layer step only enqueues kernels (no host synchronisation, no allocation, no memset
nodes), so it can be captured into a HIP graph.  Several replays, with eager work and
synchronisations between them, must reproduce the eager result bit for bit."""
import pytest
import torch

from paper_2605_11005_amd import workloads as W
from paper_2605_11005_amd.layer import run_backward, run_forward
from tests.gpu_util import gpu_layer, make_inputs

pytestmark = pytest.mark.gpu


def test_step_replays_from_a_graph_bit_for_bit():
    wl = W.DSV3.scaled(name="dsv3-graph", T=4096, d=512, f=256)
    inp = make_inputs(wl)
    dev, buf = gpu_layer(wl, inp)                      # eager reference run
    names = ("topk_idx", "topk_w", "counts", "offsets", "inv", "y", "dx", "dw1", "dw3", "dw2")
    ref = {n: getattr(buf, n).clone() for n in names}
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        run_forward(wl, dev, buf); run_backward(wl, dev, buf)      # warm-up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=s):
            run_forward(wl, dev, buf); run_backward(wl, dev, buf)
    torch.cuda.synchronize()
    for rep in range(3):
        for n in names:                                 # eager work between the replays: poison the outputs
            getattr(buf, n).fill_(3)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for n in names:
            assert torch.equal(getattr(buf, n), ref[n]), (rep, n)

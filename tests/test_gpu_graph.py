"""The layer calls only enqueue kernels on the caller's stream (no memset, copy or
synchronisation), so a forward+backward step can be captured in a HIP graph.  Replays must
reproduce the eager results bit for bit, every time, with eager work and synchronisations
between the replays."""
import numpy as np
import pytest
import torch

from paper_2502_16927_amd import binding as B
from paper_2502_16927_amd import synth
from gpu_util import DeviceLayer, add_cdac_weights

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("order", [B.ORDER_DCCA, B.ORDER_CDAC])
def test_graph_replays_equal_eager(order):
    wl = synth.small(T=1536, d=256, r=64, N=16, k=4, h=256, dtype=B.BF16, index=177)
    data = add_cdac_weights(synth.generate(wl))
    layer = DeviceLayer(wl, data, order=order)
    layer.forward(training=True)
    layer.alloc_grads()
    layer.backward()
    torch.cuda.synchronize()
    names = [n for n in ("d_w_down", "d_w_up", "d_w_gate", "d_w1", "d_w2") if order == B.ORDER_DCCA or n not in ("d_w_down", "d_w_up")]
    want = {"y": layer.y.clone(), "dx": layer.dx.clone(), **{n: layer.grads[n].clone() for n in names}}

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        layer.forward(training=True)
        layer.backward()
    for replay in range(4):
        # eager work between replays: wipe every output, run an unrelated kernel, synchronise
        layer.y.fill_(float("nan"))
        layer.dx.fill_(float("nan"))
        for n in names:
            layer.grads[n].fill_(float("nan"))
        _ = (layer.x.float() * 2).sum().item()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(layer.y, want["y"]), f"replay {replay}: y differs"
        assert torch.equal(layer.dx, want["dx"]), f"replay {replay}: dx differs"
        for n in names:
            assert torch.equal(layer.grads[n], want[n]), f"replay {replay}: {n} differs"

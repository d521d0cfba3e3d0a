"""The whole layer step (and the optimizer step) recorded into a HIP graph and replayed: every entry point launches
only kernels on the caller's stream and allocates nothing, so a captured step must reproduce the eager one bit for
bit on every replay, with other work and synchronisations in between."""
import numpy as np
import pytest
import torch

import paper_2602_11543_amd as S
from harness import DeviceLayer
from spes_workloads import CONFIGS, layer_inputs

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["cfg1", "cfg2_small"])
def test_captured_step_replays_bit_exact(device, name):
    inp = layer_inputs(CONFIGS[name])
    L = DeviceLayer(inp, device)
    losses = torch.zeros(2, dtype=torch.float32, device=device)

    def step():
        L.fwd()
        S.spes_moe_router_aux(L.shape, L.ctx, 0.01, 0.001, 1.0, losses)
        L.bwd()

    step(); torch.cuda.synchronize()
    want = [t.clone() for t in (L.y, L.dx, L.d_w_router, L.d_w_gate, L.d_w_up, L.d_w_down, losses, L.idx)]
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()                                        # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    x0 = L.x.clone()
    for rep in range(3):
        for t in (L.y, L.dx, L.d_w_router, L.d_w_gate, L.d_w_up, L.d_w_down):
            t.zero_()                                 # the program's own eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(want, (L.y, L.dx, L.d_w_router, L.d_w_gate, L.d_w_up, L.d_w_down, losses, L.idx)):
            assert torch.equal(a, b), f"replay {rep} differs"
    # a replay reads the buffers it was recorded with: new inputs in place give the eager result for those inputs
    L.x.copy_(torch.roll(x0, 1, dims=0))
    graph.replay(); torch.cuda.synchronize()
    got = [t.clone() for t in (L.y, L.dx, L.d_w_router)]
    step(); torch.cuda.synchronize()
    for a, b in zip(got, (L.y, L.dx, L.d_w_router)):
        assert torch.equal(a, b)

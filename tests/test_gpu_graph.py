"""The layer step recorded into a HIP graph and replayed: every replay must reproduce the eager result bit for bit,
also with other work between the replays and with new inputs in the same buffers (the library allocates nothing and
clears nothing with memset calls, so a capture holds kernels only)."""
import pytest
import torch

from spes_workloads import CONFIGS, layer_inputs

from harness import DeviceLayer
from paper_2602_11543_amd.layer import to_dev

pytestmark = pytest.mark.gpu


def _outputs(L):
    outs = [L.y, L.dx, L.d_w_router, L.idx, L.gate, L.count]
    if L.d_w_gate is not None:
        outs += [L.d_w_gate, L.d_w_up, L.d_w_down]
    return outs


@pytest.mark.parametrize("name", ["cfg1", "cfg2_small"])
def test_graph_replays_match_eager(name, device):
    cfg = CONFIGS[name]
    batches = [layer_inputs(cfg, micro=i) for i in range(3)]
    L = DeviceLayer(batches[0], device)
    other = DeviceLayer(layer_inputs(CONFIGS["cfg3_small"]), device)      # unrelated work between replays

    xs = [to_dev(b["x"], cfg.dtype, device) for b in batches]
    dys = [to_dev(b["dy"], cfg.dtype, device) for b in batches]

    def load(i):
        L.x.copy_(xs[i]); L.dy.copy_(dys[i])

    # eager results for each micro-batch
    want = []
    for i in range(3):
        load(i)
        L.fwd(); L.bwd(0); torch.cuda.synchronize()
        want.append([t.clone() for t in _outputs(L)])

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    load(0)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        L.fwd(); L.bwd(0)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            L.fwd(); L.bwd(0)
    torch.cuda.synchronize()

    for rep, i in enumerate([0, 1, 2, 1, 0]):
        load(i)
        for t in _outputs(L):
            t.zero_()                                                   # a replay has to write everything again
        other.fwd(); other.bwd(0)                                       # eager work of the program's own in between
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(_outputs(L), want[i]):
            assert torch.equal(got, ref), (name, rep, i)

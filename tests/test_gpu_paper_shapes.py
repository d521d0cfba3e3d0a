"""The layer shapes of the paper's own models (Sec. 4, model-configuration table) at one micro-batch of 2 x 2048
tokens, with weight gradients accumulated over two micro-batches: small-T shapes where weight traffic weighs more."""
import numpy as np
import pytest
import torch

from harness import TOL, DeviceLayer, rel_err, to_dev
from oracle import spes_oracle as O
from spes_workloads import CONFIGS, layer_inputs

from test_gpu_fullsize import _check_sampled, _routing_all_tokens

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["paper_1b", "paper_2b", "paper_7b", "paper_9b"])
def test_paper_shape_sampled(name, device):
    cfg = CONFIGS[name]
    print(f"[case] {cfg}", flush=True)
    inp = layer_inputs(cfg)
    L = DeviceLayer(inp, device)
    L.fwd(); L.bwd(); torch.cuda.synchronize()
    _check_sampled(L, inp, _routing_all_tokens(inp), n_tokens=512)


def test_two_micro_batches_accumulate(device):
    """accumulate=1 adds the second micro-batch's weight gradients to the first's; checked on one trainable expert
    and the router against the sum of the oracle's two gradients."""
    cfg = CONFIGS["paper_1b"]
    a, b = layer_inputs(cfg), layer_inputs(cfg, micro=1)
    assert not np.array_equal(a["x"], b["x"]) and np.array_equal(a["w_gate"], b["w_gate"])
    L = DeviceLayer(a, device)
    L.fwd(); L.bwd(0)
    dl_a = L.view("dlogits").cpu().numpy().astype(np.float64)
    L.x.copy_(to_dev(b["x"], cfg.dtype, device)); L.dy.copy_(to_dev(b["dy"], cfg.dtype, device))
    L.fwd(); L.bwd(1); torch.cuda.synchronize()
    dl_b = L.view("dlogits").cpu().numpy().astype(np.float64)
    tol = TOL[cfg.dtype]
    want_r = dl_a.T @ a["x"].astype(np.float64) + dl_b.T @ b["x"].astype(np.float64)
    assert rel_err(L.d_w_router.cpu().numpy(), want_r) < tol
    rt_a, rt_b = _routing_all_tokens(a), _routing_all_tokens(b)
    slot = int(np.argmin([rt_a["count"][e] + rt_b["count"][e] for e in L.trainable]))
    e = L.trainable[slot]
    ga = O.expert_weight_grads(e, rt_a, a["dy"], a["x"], a["w_gate"][e], a["w_up"][e], a["w_down"][e])
    gb = O.expert_weight_grads(e, rt_b, b["dy"], b["x"], b["w_gate"][e], b["w_up"][e], b["w_down"][e])
    for got, x, y in zip((L.d_w_gate[slot], L.d_w_up[slot], L.d_w_down[slot]), ga, gb):
        assert rel_err(got.cpu().numpy(), x + y) < tol

"""GPU parity of the stand-alone backward of the combine (spes_moe_grad_scatter) against the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import spes_oracle as O
from spes_workloads import CONFIGS, custom_config, layer_inputs, bf16_round

from harness import TOL, DeviceLayer, rel_err

pytestmark = pytest.mark.gpu


def _case(inp, device):
    cfg = inp["cfg"]
    L = DeviceLayer(inp, device)
    L.fwd()
    dyp, dgate = L.grad_scatter()
    torch.cuda.synchronize()
    fwd = O.moe_forward(inp["x"], inp["w_router"], inp["router_bias"], inp["w_gate"], inp["w_up"], inp["w_down"], cfg.k, cfg.renorm)
    assert np.array_equal(L.view("perm").cpu().numpy(), fwd["perm"])
    # chain rule on Eq. 2: the routed row of pair (t, j) receives gate[t,j] * dy[t]; the gate receives <dy[t], yp[t,j]>
    t_of, j_of = fwd["perm"] // cfg.k, fwd["perm"] % cfg.k
    want_dyp = fwd["gate"][t_of, j_of][:, None] * inp["dy"].astype(np.float64)[t_of]
    want_dgate = np.einsum("td,tjd->tj", inp["dy"].astype(np.float64), fwd["yp"])
    got_dyp = L.host(dyp)
    tol = TOL[cfg.dtype]
    assert rel_err(got_dyp, want_dyp) <= tol
    if cfg.dtype == "bf16":      # a product rounded once: one bf16 ulp of the exact product, element by element
        assert np.all(np.abs(got_dyp - want_dyp) <= 2.0 ** -8 * np.abs(want_dyp) + 1e-30)
    assert rel_err(dgate.cpu().numpy(), want_dgate) <= tol
    return L


@pytest.mark.parametrize("name", ["cfg1", "cfg2_small", "cfg3_small", "cfg4_small"])
def test_grad_scatter_parity(name, device):
    print(f"[case] grad scatter {name}", flush=True)
    _case(layer_inputs(CONFIGS[name]), device)


@pytest.mark.parametrize("kw", [
    dict(T=1, d=64, M=4, f=64, k=2),
    dict(T=130, d=64, M=6, f=56, k=6, dtype="bf16"),                   # k outside the unrolled cases
    dict(T=257, d=136, M=64, f=72, k=3, dtype="bf16"),                  # a feature size that is not a multiple of the block
    dict(T=70, d=4104, M=8, f=64, k=4, dtype="bf16"),                   # more than one pass over the feature axis, ragged
    dict(T=90, d=1032, M=8, f=64, k=1),
])
def test_grad_scatter_edge_cases(kw, device):
    kw = dict(kw); kw.setdefault("router_sigma", 0.3)
    print(f"[case] grad scatter {kw}", flush=True)
    _case(layer_inputs(custom_config(**kw)), device)

"""GPU parity of spes_moe_fwd / spes_moe_bwd against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import spes_oracle as O
from spes_workloads import CONFIGS, custom_config, layer_inputs

from harness import TOL, DeviceLayer, check_routing, rel_err

pytestmark = pytest.mark.gpu


def _full_parity(inp, device, label):
    cfg = inp["cfg"]
    tol = TOL[cfg.dtype]
    L = DeviceLayer(inp, device)
    print(f"[case] {label} {cfg}", flush=True)
    L.fwd(); L.bwd(); torch.cuda.synchronize()
    fwd = O.moe_forward(inp["x"], inp["w_router"], inp["router_bias"], inp["w_gate"], inp["w_up"], inp["w_down"], cfg.k, cfg.renorm)
    bwd = O.moe_backward(fwd, inp["dy"], inp["x"], inp["w_router"], inp["w_gate"], inp["w_up"], inp["w_down"], cfg.renorm,
                         wgrad_experts=L.trainable)
    check_routing(L, fwd)
    errs = dict(gate=rel_err(L.host(L.gate), fwd["gate"]), y=rel_err(L.host(L.y), fwd["y"]),
                dx=rel_err(L.host(L.dx), bwd["dx"]), d_w_router=rel_err(L.host(L.d_w_router), bwd["d_w_router"]))
    for slot, e in enumerate(L.trainable):
        errs[f"dWg[{e}]"] = rel_err(L.host(L.d_w_gate[slot]), bwd["d_w_gate"][e])
        errs[f"dWu[{e}]"] = rel_err(L.host(L.d_w_up[slot]), bwd["d_w_up"][e])
        errs[f"dWd[{e}]"] = rel_err(L.host(L.d_w_down[slot]), bwd["d_w_down"][e])
    worst = max(errs, key=errs.get)
    print(f"  worst {worst} = {errs[worst]:.3e} (tol {tol})", flush=True)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, bad
    return L, fwd, bwd


@pytest.mark.parametrize("name", ["cfg1", "cfg1_bf16", "cfg2_f32", "cfg2_small", "cfg3_small", "cfg4_small"])
def test_layer_parity(name, device):
    _full_parity(layer_inputs(CONFIGS[name]), device, name)


@pytest.mark.parametrize("kw", [
    dict(T=1, d=64, M=4, f=64, k=2),                                    # a single token
    dict(T=67, d=72, M=1, f=40, k=1, n_trainable=1),                    # one expert: a plain SwiGLU FFN
    dict(T=130, d=64, M=6, f=56, k=6, n_trainable=3),                   # k = M: dense mixture
    dict(T=257, d=136, M=64, f=72, k=3, n_trainable=7, trainable="random"),   # more experts than most tiles have rows
    dict(T=200, d=64, M=8, f=64, k=1, bias="normal", bias_scale=8.0),    # nearly every token to one expert, several empty
    # collapsed routing: the top probability is 1 to within fp32 rounding, and the router gradient (about 1e-8 of the
    # gate gradient) survives only because the gating backward never forms 1 - p by subtraction
    dict(T=200, d=64, M=8, f=64, k=1, bias="normal", bias_scale=30.0),
    dict(T=200, d=64, M=8, f=64, k=2, bias="normal", bias_scale=30.0),
    dict(T=200, d=64, M=8, f=64, k=2, renorm=1, bias="normal", bias_scale=30.0),
    dict(T=333, d=264, M=16, f=200, k=4, renorm=1, dtype="bf16", n_trainable=5, trainable="random", router_sigma=0.05),
    dict(T=96, d=64, M=8, f=64, k=2, n_trainable=0),                    # nothing trainable: no weight-grad buffers at all
    # the same corners through the matrix-core path (bf16): contraction lengths of one and two K-tiles with and
    # without a tail, two passes of one tile each, experts with fewer rows than one k-tile or none at all
    dict(T=1, d=64, M=4, f=64, k=2, dtype="bf16"),
    dict(T=67, d=72, M=1, f=40, k=1, n_trainable=1, dtype="bf16"),
    dict(T=130, d=64, M=6, f=56, k=6, n_trainable=3, dtype="bf16"),
    dict(T=257, d=136, M=64, f=72, k=3, n_trainable=7, trainable="random", dtype="bf16"),
    dict(T=200, d=128, M=8, f=128, k=1, bias="normal", bias_scale=8.0, dtype="bf16"),
    dict(T=200, d=128, M=8, f=128, k=2, bias="normal", bias_scale=30.0, dtype="bf16"),
    dict(T=96, d=8, M=8, f=8, k=2, n_trainable=8, dtype="bf16"),        # the smallest feature sizes the library takes
    dict(T=300, d=192, M=12, f=320, k=2, renorm=1, n_trainable=0, dtype="bf16"),
    # outputs wide enough for the grouped tile order (at least 12 column tiles), with a ragged last group of row tiles
    dict(T=700, d=64, M=5, f=1600, k=2, n_trainable=2, dtype="bf16"),
    dict(T=700, d=3200, M=5, f=64, k=2, n_trainable=2, dtype="bf16"),
    # a last column tile that is at most half full runs as a launch of its own on the half-width tile: exactly half
    # (d and f = 128 beyond a multiple of 256), and a quarter (64 beyond)
    dict(T=600, d=384, M=6, f=640, k=2, n_trainable=2, dtype="bf16"),
    dict(T=600, d=320, M=6, f=576, k=2, renorm=1, n_trainable=3, trainable="random", dtype="bf16"),
    # few tiles and outputs a multiple of 256 wide: whole launches on the half-width tile, the SwiGLU-backward one included
    dict(T=1024, d=256, M=4, f=512, k=2, n_trainable=2, dtype="bf16"),
    # fp32 path with enough 64-row tiles for the tallest of its three tile heights (the cases above use the shorter two)
    dict(T=2048, d=128, M=4, f=512, k=2, n_trainable=2),
])
def test_layer_edge_cases(kw, device):
    kw = dict(kw); kw.setdefault("router_sigma", 0.3)
    inp = layer_inputs(custom_config(**kw))
    L, fwd, _ = _full_parity(inp, device, "edge")
    if kw.get("bias_scale", 0) >= 8:
        assert (fwd["count"] == 0).any()


def test_mask_does_not_change_other_results(device):
    inp = layer_inputs(CONFIGS["cfg2_small"])
    L = DeviceLayer(inp, device)
    L.fwd(); L.bwd(); torch.cuda.synchronize()
    base = dict(dx=L.dx.clone(), dwr=L.d_w_router.clone(),
                g={e: L.d_w_gate[s].clone() for s, e in enumerate(L.trainable)},
                d={e: L.d_w_down[s].clone() for s, e in enumerate(L.trainable)})
    keep = L.trainable[::2]
    mask = np.zeros(L.cfg.M, dtype=np.uint8); mask[keep] = 1; mask[[e for e in range(L.cfg.M) if e not in L.trainable][:3]] = 1
    L.set_mask(mask)
    assert L.d_w_gate.shape[0] == int(mask.sum())          # buffers exist for trainable experts only
    L.bwd(); torch.cuda.synchronize()
    assert torch.equal(L.dx, base["dx"]) and torch.equal(L.d_w_router, base["dwr"])
    for s, e in enumerate(L.trainable):
        if e in keep:
            assert torch.equal(L.d_w_gate[s], base["g"][e]) and torch.equal(L.d_w_down[s], base["d"][e])


def test_accumulate_and_determinism(device):
    inp = layer_inputs(CONFIGS["cfg1"])
    L = DeviceLayer(inp, device)
    L.fwd(); L.bwd(0); torch.cuda.synchronize()
    once = [t.clone() for t in (L.y, L.dx, L.d_w_router, L.d_w_gate, L.d_w_up, L.d_w_down)]
    L.fwd(); L.bwd(0); torch.cuda.synchronize()
    for a, b in zip(once, (L.y, L.dx, L.d_w_router, L.d_w_gate, L.d_w_up, L.d_w_down)):
        assert torch.equal(a, b)                            # bit-reproducible
    L.bwd(1); torch.cuda.synchronize()
    for a, b in zip(once[2:], (L.d_w_router, L.d_w_gate, L.d_w_up, L.d_w_down)):
        assert torch.equal(2 * a, b)                        # x + x is exact
    assert torch.equal(once[1], L.dx)


def test_argument_errors(device):
    import paper_2602_11543_amd as S
    inp = layer_inputs(custom_config(T=8, d=64, M=4, f=64, k=2))
    L = DeviceLayer(inp, device)
    bad = S.moe_shape(8, 64, 4, 64, 5, 0, 0)                # top_k > n_experts
    assert S.spes_moe_ctx_bytes(bad) == 0
    with pytest.raises(S.SpesError, match="invalid"):
        S.spes_moe_fwd(bad, L.x, L.w_router, None, L.w_gate, L.w_up, L.w_down, L.y, L.idx, L.gate, L.count, L.ctx)
    with pytest.raises(S.SpesError, match="unsupported"):
        S.spes_moe_fwd(S.moe_shape(8, 60, 4, 64, 2, 0, 0), L.x, L.w_router, None, L.w_gate, L.w_up, L.w_down, L.y, L.idx,
                       L.gate, L.count, L.ctx)
    with pytest.raises(S.SpesError, match="aligned"):
        S.spes_moe_fwd(L.shape, L.x.view(-1)[1:], L.w_router, None, L.w_gate, L.w_up, L.w_down, L.y, L.idx, L.gate, L.count, L.ctx)
    with pytest.raises(S.SpesError, match="invalid"):
        S.spes_moe_bwd(L.shape, L.dy, L.x, L.w_router, L.w_gate, L.w_up, L.w_down, L.ctx, L.mask, L.dx, L.d_w_router,
                       None, L.d_w_up, L.d_w_down)


@pytest.mark.gpu
def test_mfma_reference_loop_runs_and_counts_its_work():
    """The benchmark's register-resident MFMA loop: launches, reports its operation count, and writes its sink."""
    import paper_2602_11543_amd as S
    dev = torch.device("cuda:0")
    data = (torch.randn(32768, device=dev) * 0.02).to(torch.bfloat16)
    sink = torch.full((8,), float("nan"), device=dev)
    flop = S.spes_ref_mfma_rate(data, 8, 10, sink)
    torch.cuda.synchronize()
    assert flop == 8 * 4 * 10 * 64 * 2.0 * 16 * 16 * 32
    assert bool(torch.isfinite(sink).all())

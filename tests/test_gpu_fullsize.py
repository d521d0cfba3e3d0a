"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

Routing is compared bit for bit for every token.  The gate gradient, dlogits and the router weight gradient are
compared for every token with the oracle's own values (its expert forward run one expert at a time), the weight
gradients of every trainable expert (the most loaded included) one expert at a time, and y and dx on sampled tokens
(tokens are independent there).  The 2B-shaped layer is additionally checked in full.
"""
import numpy as np
import pytest
import torch

import paper_2602_11543_amd as S
from oracle import spes_oracle as O
from spes_workloads import CONFIGS, layer_inputs, merge_inputs, bf16_round

from harness import TOL, DeviceLayer, rel_err, storage_ulp_excess, to_dev

pytestmark = pytest.mark.gpu


def _routing_all_tokens(inp):
    cfg = inp["cfg"]
    s = O.router_logits(inp["x"], inp["w_router"], inp["router_bias"])
    p = O.softmax(s)
    idx = O.top_k(s, cfg.k)
    gate = O.gates(p, idx, cfg.renorm)
    count, offset, perm, inv = O.routing_tables(idx, cfg.M)
    return dict(logits=s, p=p, idx=idx, gate=gate, count=count, offset=offset, perm=perm, inv=inv)


def _check_sampled(L, inp, rt, n_tokens=768, n_experts=None, seed=0):
    cfg = inp["cfg"]
    tol = TOL[cfg.dtype]
    rng = np.random.default_rng(seed)
    # ---- integer routing results, every token ----
    assert np.array_equal(L.idx.cpu().numpy(), rt["idx"])
    assert np.array_equal(L.count.cpu().numpy(), rt["count"])
    assert np.array_equal(L.view("offset").cpu().numpy(), rt["offset"])
    assert np.array_equal(L.view("perm").cpu().numpy(), rt["perm"])
    assert np.array_equal(L.view("inv").cpu().numpy(), rt["inv"])
    assert rel_err(L.gate.cpu().numpy(), rt["gate"]) <= 1e-5
    # the dispatched copy of x, every row: a byte-exact gather through the (oracle-checked) permutation
    xp = L.permuted()
    tok = torch.from_numpy(rt["perm"] // cfg.k).to(L.dev).long()
    for r0 in range(0, tok.numel(), 1 << 16):
        assert torch.equal(xp[r0:r0 + (1 << 16)].view(torch.uint8), L.x[tok[r0:r0 + (1 << 16)]].view(torch.uint8)), "permuted input differs"
    del xp
    # ---- sampled tokens: y, dx, dgate, dlogits ----
    pick = np.sort(rng.choice(cfg.T, size=min(n_tokens, cfg.T), replace=False))
    fwd = O.moe_forward(inp["x"][pick], inp["w_router"], inp["router_bias"], inp["w_gate"], inp["w_up"], inp["w_down"],
                        cfg.k, cfg.renorm)
    assert np.array_equal(fwd["idx"], rt["idx"][pick])
    bwd = O.moe_backward(fwd, inp["dy"][pick], inp["x"][pick], inp["w_router"], inp["w_gate"], inp["w_up"], inp["w_down"],
                         cfg.renorm, wgrad_experts=[])
    errs = dict(y=rel_err(L.host(L.y)[pick], fwd["y"]), dx=rel_err(L.host(L.dx)[pick], bwd["dx"]),
                dgate=rel_err(L.view("dgate").cpu().numpy()[pick], bwd["dgate"]),
                dlogits=rel_err(L.view("dlogits").cpu().numpy()[pick], bwd["dlogits"]))
    # ---- gate gradient, dlogits and the router weight gradient for every token: the oracle's expert forward, one
    # expert at a time (no per-pair intermediate is kept), then its gating backward and dlogits^T x ----
    dgate = np.full((cfg.T, cfg.k), np.nan)
    for e in range(cfg.M):
        t_e, j_e, v = O.expert_gate_grads(e, rt, inp["dy"], inp["x"], inp["w_gate"][e], inp["w_up"][e], inp["w_down"][e])
        dgate[t_e, j_e] = v
    assert not np.isnan(dgate).any()
    dl = O.gating_backward(rt["p"], rt["idx"], rt["gate"], dgate, cfg.renorm)
    errs["dgate_all"] = rel_err(L.view("dgate").cpu().numpy(), dgate)
    errs["dlogits_all"] = rel_err(L.view("dlogits").cpu().numpy(), dl)
    errs["d_w_router"] = rel_err(L.host(L.d_w_router), dl.T @ inp["x"].astype(np.float64))
    del dgate, dl
    # ---- weight gradients of the trainable experts, one at a time: all of them, or the n_experts with the longest
    # and the n_experts with the shortest contraction (the most and the least loaded) ----
    order = sorted(range(len(L.trainable)), key=lambda s: rt["count"][L.trainable[s]])
    slots = order if n_experts is None or 2 * n_experts >= len(order) else order[:n_experts] + order[-n_experts:]
    print(f"  weight gradients of experts {[L.trainable[s] for s in slots]} with {[int(rt['count'][L.trainable[s]]) for s in slots]} rows", flush=True)
    for slot in slots:
        e = L.trainable[slot]
        dwg, dwu, dwd = O.expert_weight_grads(e, rt, inp["dy"], inp["x"], inp["w_gate"][e], inp["w_up"][e], inp["w_down"][e])
        errs[f"dWg[{e}]"] = rel_err(L.host(L.d_w_gate[slot]), dwg)
        errs[f"dWu[{e}]"] = rel_err(L.host(L.d_w_up[slot]), dwu)
        errs[f"dWd[{e}]"] = rel_err(L.host(L.d_w_down[slot]), dwd)
    print("  " + ", ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, bad


@pytest.mark.parametrize("name", ["cfg2", "cfg3", "cfg4"])
def test_full_size_sampled(name, device):
    cfg = CONFIGS[name]
    print(f"[case] full size {cfg}", flush=True)
    inp = layer_inputs(cfg)
    L = DeviceLayer(inp, device)
    L.fwd(); L.bwd(); torch.cuda.synchronize()
    rt = _routing_all_tokens(inp)
    print(f"  redraw fraction {inp['redraw_fraction']:.3f}, max/mean load {rt['count'].max() / rt['count'].mean():.2f}", flush=True)
    if name == "cfg3":
        assert rt["count"].max() >= 4 * rt["count"].mean()        # the heavy-tailed bias does its job
    _check_sampled(L, inp, rt)


def test_full_size_cfg2_every_element(device):
    cfg = CONFIGS["cfg2"]
    print(f"[case] full oracle {cfg}", flush=True)
    inp = layer_inputs(cfg)
    L = DeviceLayer(inp, device)
    L.fwd(); L.bwd(); torch.cuda.synchronize()
    fwd = O.moe_forward(inp["x"], inp["w_router"], inp["router_bias"], inp["w_gate"], inp["w_up"], inp["w_down"], cfg.k, cfg.renorm)
    bwd = O.moe_backward(fwd, inp["dy"], inp["x"], inp["w_router"], inp["w_gate"], inp["w_up"], inp["w_down"], cfg.renorm,
                         wgrad_experts=L.trainable)
    assert np.array_equal(L.idx.cpu().numpy(), fwd["idx"]) and np.array_equal(L.view("perm").cpu().numpy(), fwd["perm"])
    errs = dict(y=rel_err(L.host(L.y), fwd["y"]), dx=rel_err(L.host(L.dx), bwd["dx"]),
                d_w_router=rel_err(L.host(L.d_w_router), bwd["d_w_router"]))
    for slot, e in enumerate(L.trainable):
        errs[f"dWg[{e}]"] = rel_err(L.host(L.d_w_gate[slot]), bwd["d_w_gate"][e])
        errs[f"dWu[{e}]"] = rel_err(L.host(L.d_w_up[slot]), bwd["d_w_up"][e])
        errs[f"dWd[{e}]"] = rel_err(L.host(L.d_w_down[slot]), bwd["d_w_down"][e])
    worst = max(errs, key=errs.get)
    print(f"  worst {worst} = {errs[worst]:.3e}", flush=True)
    assert errs[worst] <= TOL["bf16"], errs


def test_full_size_merge_then_layer(device):
    """16 node copies of the 64-expert layer are merged (three matrices), then one fwd+bwd runs on the merged weights."""
    cfg = CONFIGS["cfg5"]
    print(f"[case] merge sweep + layer {cfg}", flush=True)
    inp = layer_inputs(cfg)
    merged = {}
    slot = None
    for mi_seed, wname in enumerate(("w_gate", "w_up", "w_down")):
        base = inp[wname].reshape(cfg.M, -1)
        mi = merge_inputs(cfg.M, base.shape[1], 16, 16, "bf16", seed=cfg.seed, base=base, need_zero_and_single=True)
        slot = mi["slot"]
        dst = to_dev(mi["base"], "bf16", device)
        stores = [to_dev(s, "bf16", device) for s in mi["stores"]]
        cnt = torch.empty(cfg.M, dtype=torch.int32, device=device)
        S.spes_expert_merge(cfg.M, base.shape[1], S.SPES_BF16, stores, mi["slot"], mi["node_weight"], dst, cnt)
        torch.cuda.synchronize()
        got = dst.float().cpu().numpy()
        assert np.array_equal(cnt.cpu().numpy(), mi["trainer_count"]) and int(mi["trainer_count"].sum()) == 256
        want, _ = O.sync_merge(mi["base"], mi["stores"], mi["slot"], mi["node_weight"])
        mag = np.abs(mi["base"]).astype(np.float32)
        for i, st in enumerate(mi["stores"]):
            for j in np.nonzero(mi["slot"][i] >= 0)[0]:
                mag[j] = np.maximum(mag[j], np.abs(st[mi["slot"][i, j]]))
        assert storage_ulp_excess(got, want, mag, "bf16") <= 0          # one bf16 ulp from the rounded fp64 mean
        for j in np.nonzero(mi["trainer_count"] == 0)[0]:
            assert np.array_equal(got[j], mi["base"][j])
        for j in np.nonzero(mi["trainer_count"] == 1)[0]:
            i = int(np.nonzero(mi["slot"][:, j] >= 0)[0][0])
            assert np.array_equal(got[j], mi["stores"][i][mi["slot"][i, j]])
        merged[wname] = got.reshape(inp[wname].shape)
        del stores, dst
    inp2 = dict(inp)
    inp2.update(merged)
    inp2["trainable_mask"] = (slot[0] >= 0).astype(np.uint8)       # node 0's experts
    # the merged weights move the router margins of nobody (the router is untouched), so the tokens stay valid
    L = DeviceLayer(inp2, device)
    L.fwd(); L.bwd(); torch.cuda.synchronize()
    _check_sampled(L, inp2, _routing_all_tokens(inp2), n_tokens=512)

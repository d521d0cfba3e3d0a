"""Pins for the fp64 oracle of the routed SwiGLU layer (CPU only).

Each test ties the oracle to something other than itself: a hand-derived closed
form, a brute-force evaluation with Python loops, torch's autograd on an
independently written dense formulation, finite differences, or a special case
that reduces to a textbook routine.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import spes_oracle as O
from spes_workloads import custom_config, layer_inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _inputs(**kw):
    return layer_inputs(custom_config(**kw))


def _fwd(inp, keep=True):
    c = inp["cfg"]
    return O.moe_forward(inp["x"], inp["w_router"], inp["router_bias"], inp["w_gate"], inp["w_up"],
                         inp["w_down"], c.k, c.renorm, keep=keep)


def _bwd(inp, fwd):
    c = inp["cfg"]
    return O.moe_backward(fwd, inp["dy"], inp["x"], inp["w_router"], inp["w_gate"], inp["w_up"], inp["w_down"], c.renorm)


# ------------------------------------------------------------------ closed form

def _golden():
    vals = {}
    with open(os.path.join(GOLDEN, "closed_form_layer.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            name, v = line.split()
            vals[name] = float(v)
    return vals


@pytest.mark.parametrize("renorm", [0, 1])
def test_closed_form_example(renorm):
    g = _golden()
    ln3 = math.log(3.0)
    x = np.array([[1.0]]); w_r = np.zeros((2, 1)); bias = np.array([ln3, 0.0])
    wg = np.array([[[ln3]], [[0.3]]]); wu = np.array([[[2.0]], [[0.7]]]); wd = np.array([[[5.0]], [[-1.0]]])
    fwd = O.moe_forward(x, w_r, bias, wg, wu, wd, 1, renorm)
    assert fwd["idx"].tolist() == [[0]]
    np.testing.assert_allclose(fwd["p"], [[0.75, 0.25]], rtol=1e-15)
    np.testing.assert_allclose(fwd["y"][0, 0], g["y_renorm" if renorm else "y_norenorm"], rtol=1e-14)
    bwd = O.moe_backward(fwd, np.array([[1.0]]), x, w_r, wg, wu, wd, renorm)
    np.testing.assert_allclose(bwd["dgate"][0, 0], g["dgate"], rtol=1e-14)
    if renorm:
        np.testing.assert_allclose(bwd["dlogits"], 0.0, atol=1e-15)
    else:
        np.testing.assert_allclose(bwd["d_w_down"][0][0, 0], g["dW_d_norenorm"], rtol=1e-14)
        np.testing.assert_allclose(bwd["d_w_up"][0][0, 0], g["dW_u_norenorm"], rtol=1e-14)
        np.testing.assert_allclose(bwd["dlogits"][0], [g["dlogit0_norenorm"], -g["dlogit0_norenorm"]], rtol=1e-14)


# ------------------------------------------------------------------ routing

def _brute_topk(row, k):
    """Selection by repeated scan: the largest remaining score, the lowest index among equals."""
    left = list(range(len(row)))
    out = []
    for _ in range(k):
        best = left[0]
        for e in left[1:]:
            if row[e] > row[best]:
                best = e
        out.append(best)
        left.remove(best)
    return out


def test_topk_bruteforce_and_ties():
    rng = np.random.default_rng(0)
    s = rng.standard_normal((40, 7))
    s[3, 2] = s[3, 5] = s[3].max() + 1.0       # a tie for first place
    s[4, :] = 0.25                             # all equal
    for k in (1, 3, 7):
        idx = O.top_k(s, k)
        for t in range(s.shape[0]):
            assert idx[t].tolist() == _brute_topk(s[t], k)
    assert O.top_k(s, 2)[3].tolist() == [2, 5]
    assert O.top_k(s, 3)[4].tolist() == [0, 1, 2]


def test_routing_tables_bruteforce_and_invariants():
    rng = np.random.default_rng(1)
    T, M, k = 37, 6, 3
    idx = np.stack([rng.permutation(M)[:k] for _ in range(T)]).astype(np.int32)
    count, offset, perm, inv = O.routing_tables(idx, M)
    # brute force: walk experts, then flat pair index ascending
    rows = []
    for e in range(M):
        for r in range(T * k):
            if idx.reshape(-1)[r] == e:
                rows.append(r)
    assert perm.tolist() == rows
    assert count.sum() == T * k and offset[0] == 0 and offset[-1] == T * k
    assert np.all(np.diff(offset) == count)
    assert np.array_equal(inv[perm], np.arange(T * k)) and np.array_equal(perm[inv], np.arange(T * k))
    for e in range(M):
        seg = perm[offset[e]:offset[e + 1]]
        assert np.all(idx.reshape(-1)[seg] == e) and np.all(np.diff(seg) > 0)


def test_routing_empty_expert():
    idx = np.array([[0, 2], [2, 0], [0, 2]], dtype=np.int32)
    count, offset, perm, inv = O.routing_tables(idx, 4)
    assert count.tolist() == [3, 0, 3, 0] and offset.tolist() == [0, 3, 3, 6, 6]
    assert perm.tolist() == [0, 3, 4, 1, 2, 5]


def test_softmax_against_scipy():
    from scipy.special import softmax as sp_softmax
    s = np.random.default_rng(2).standard_normal((11, 9)) * 30.0
    np.testing.assert_allclose(O.softmax(s), sp_softmax(s, axis=1), rtol=1e-13)


# ------------------------------------------------------------------ forward

def _python_loop_layer(inp):
    """The definition with scalar Python arithmetic only (tiny shapes)."""
    c = inp["cfg"]
    x, wr, wg, wu, wd = (inp[n].astype(np.float64) for n in ("x", "w_router", "w_gate", "w_up", "w_down"))
    bias = inp["router_bias"]
    y = np.zeros((c.T, c.d))
    for t in range(c.T):
        s = [sum(x[t, i] * wr[e, i] for i in range(c.d)) + (float(bias[e]) if bias is not None else 0.0) for e in range(c.M)]
        mx = max(s)
        ex = [math.exp(v - mx) for v in s]
        p = [v / sum(ex) for v in ex]
        sel = _brute_topk(s, c.k)
        norm = sum(p[e] for e in sel) if c.renorm else 1.0
        for e in sel:
            hvec = []
            for r in range(c.f):
                a = sum(wg[e, r, i] * x[t, i] for i in range(c.d))
                b = sum(wu[e, r, i] * x[t, i] for i in range(c.d))
                hvec.append(a / (1.0 + math.exp(-a)) * b)
            for i in range(c.d):
                y[t, i] += p[e] / norm * sum(wd[e, i, r] * hvec[r] for r in range(c.f))
    return y


@pytest.mark.parametrize("renorm,bias", [(0, "none"), (1, "normal")])
def test_forward_python_loops(renorm, bias):
    inp = _inputs(T=6, d=5, M=4, f=3, k=2, renorm=renorm, bias=bias, bias_scale=0.5, router_sigma=0.5)
    np.testing.assert_allclose(_fwd(inp)["y"], _python_loop_layer(inp), rtol=1e-12, atol=1e-15)


def test_single_expert_is_plain_swiglu_ffn():
    inp = _inputs(T=9, d=8, M=1, f=12, k=1, n_trainable=1)
    xt = torch.from_numpy(inp["x"]).double()
    wg, wu, wd = (torch.from_numpy(inp[n][0]).double() for n in ("w_gate", "w_up", "w_down"))
    ref = torch.nn.functional.linear(torch.nn.functional.silu(torch.nn.functional.linear(xt, wg))
                                     * torch.nn.functional.linear(xt, wu), wd)
    fwd = _fwd(inp)
    np.testing.assert_allclose(fwd["gate"], 1.0, rtol=1e-15)
    np.testing.assert_allclose(fwd["y"], ref.numpy(), rtol=1e-12, atol=1e-18)


def test_k_equals_M_is_dense_softmax_mixture():
    inp = _inputs(T=10, d=6, M=5, f=7, k=5, router_sigma=0.7)
    x = torch.from_numpy(inp["x"]).double()
    p = torch.softmax(x @ torch.from_numpy(inp["w_router"]).double().T, dim=1)
    ref = torch.zeros(10, 6, dtype=torch.float64)
    for e in range(5):
        wg, wu, wd = (torch.from_numpy(inp[n][e]).double() for n in ("w_gate", "w_up", "w_down"))
        ref += p[:, e:e + 1] * ((torch.nn.functional.silu(x @ wg.T) * (x @ wu.T)) @ wd.T)
    np.testing.assert_allclose(_fwd(inp)["y"], ref.numpy(), rtol=1e-12, atol=1e-18)


def test_identical_experts_with_renorm_equal_one_expert():
    # renormalised gates sum to one, so M copies of one FFN reproduce that FFN (Sec. 4, upcycled model)
    inp = _inputs(T=12, d=8, M=6, f=10, k=3, renorm=1, router_sigma=0.6)
    for n in ("w_gate", "w_up", "w_down"):
        inp[n][:] = inp[n][0]
    _, _, _, ref = O.expert_forward(inp["x"], inp["w_gate"][0], inp["w_up"][0], inp["w_down"][0])
    np.testing.assert_allclose(_fwd(inp)["y"], ref, rtol=1e-12, atol=1e-18)


def test_gate_properties():
    inp = _inputs(T=50, d=16, M=8, f=4, k=3, renorm=1, router_sigma=0.5)
    fwd = _fwd(inp)
    np.testing.assert_allclose(fwd["gate"].sum(1), 1.0, rtol=1e-14)
    assert np.all(np.diff(fwd["gate"], axis=1) <= 0)          # descending score order
    inp0 = _inputs(T=50, d=16, M=8, f=4, k=3, renorm=0, router_sigma=0.5)
    f0 = _fwd(inp0)
    np.testing.assert_allclose(f0["gate"], np.take_along_axis(f0["p"], f0["idx"].astype(np.int64), 1))
    assert np.all(f0["gate"].sum(1) < 1.0)


# ------------------------------------------------------------------ backward

def _torch_dense_layer(inp, idx):
    """Independent dense formulation: every expert on every token, one-hot selection mask, autograd."""
    c = inp["cfg"]
    leaves = {n: torch.from_numpy(inp[n]).double().requires_grad_(True) for n in ("x", "w_router", "w_gate", "w_up", "w_down")}
    x = leaves["x"]
    s = x @ leaves["w_router"].T
    if inp["router_bias"] is not None:
        s = s + torch.from_numpy(inp["router_bias"]).double()
    p = torch.softmax(s, dim=1)
    sel = torch.zeros(c.T, c.M, dtype=torch.float64)
    sel.scatter_(1, torch.from_numpy(idx.astype(np.int64)), 1.0)
    g = p * sel
    if c.renorm:
        g = g / g.sum(dim=1, keepdim=True)
    a = torch.einsum("td,efd->tef", x, leaves["w_gate"])
    b = torch.einsum("td,efd->tef", x, leaves["w_up"])
    yp = torch.einsum("tef,edf->ted", torch.nn.functional.silu(a) * b, leaves["w_down"])
    y = (g[:, :, None] * yp).sum(dim=1)
    return y, leaves


@pytest.mark.parametrize("renorm,bias,k", [(0, "normal", 2), (1, "none", 3), (0, "none", 1), (1, "gumbel", 1)])
def test_backward_against_autograd_dense_formulation(renorm, bias, k):
    inp = _inputs(T=23, d=10, M=6, f=9, k=k, renorm=renorm, bias=bias, bias_scale=0.5, router_sigma=0.6)
    fwd = _fwd(inp)
    bwd = _bwd(inp, fwd)
    y, leaves = _torch_dense_layer(inp, fwd["idx"])
    np.testing.assert_allclose(fwd["y"], y.detach().numpy(), rtol=1e-12, atol=1e-16)
    y.backward(torch.from_numpy(inp["dy"]).double())
    np.testing.assert_allclose(bwd["dx"], leaves["x"].grad.numpy(), rtol=1e-10, atol=1e-14)
    np.testing.assert_allclose(bwd["d_w_router"], leaves["w_router"].grad.numpy(), rtol=1e-10, atol=1e-14)
    for e in range(6):
        np.testing.assert_allclose(bwd["d_w_gate"][e], leaves["w_gate"].grad[e].numpy(), rtol=1e-10, atol=1e-14)
        np.testing.assert_allclose(bwd["d_w_up"][e], leaves["w_up"].grad[e].numpy(), rtol=1e-10, atol=1e-14)
        np.testing.assert_allclose(bwd["d_w_down"][e], leaves["w_down"].grad[e].numpy(), rtol=1e-10, atol=1e-14)


@pytest.mark.parametrize("renorm", [0, 1])
def test_backward_finite_differences(renorm):
    """Central differences of L = <dy, y> along random directions in every differentiable input."""
    inp = _inputs(T=17, d=12, M=5, f=8, k=2, renorm=renorm, router_sigma=0.5)
    fwd = _fwd(inp)
    bwd = _bwd(inp, fwd)
    dy = inp["dy"].astype(np.float64)
    rng = np.random.default_rng(5)
    grads = dict(x=bwd["dx"], w_router=bwd["d_w_router"],
                 w_gate=np.stack([bwd["d_w_gate"][e] for e in range(5)]),
                 w_up=np.stack([bwd["d_w_up"][e] for e in range(5)]),
                 w_down=np.stack([bwd["d_w_down"][e] for e in range(5)]))
    for name, g in grads.items():
        base = inp[name].astype(np.float64)
        v = rng.standard_normal(base.shape)
        eps = 1e-6 * np.abs(base).max()
        vals = []
        for sgn in (+1, -1):
            trial = dict(inp); trial[name] = base + sgn * eps * v
            f = _fwd(trial, keep=False)
            assert np.array_equal(f["idx"], fwd["idx"])          # the margin keeps the selection fixed
            vals.append(np.sum(dy * f["y"]))
        fd = (vals[0] - vals[1]) / (2 * eps)
        an = np.sum(g * v)
        assert abs(fd - an) <= 1e-6 * max(abs(an), 1e-12), (name, fd, an)


def test_gating_backward_properties():
    rng = np.random.default_rng(7)
    T, M, k = 30, 9, 4
    s = rng.standard_normal((T, M))
    p = O.softmax(s); idx = O.top_k(s, k)
    dgate = rng.standard_normal((T, k))
    for renorm in (0, 1):
        g = O.gates(p, idx, renorm)
        dl = O.gating_backward(p, idx, g, dgate, renorm)
        np.testing.assert_allclose(dl.sum(1), 0.0, atol=1e-14)     # softmax is shift-invariant
    # renormalised gates are a softmax over the selected logits alone
    g = O.gates(p, idx, 1)
    closed = np.zeros((T, M))
    np.put_along_axis(closed, idx.astype(np.int64), g * (dgate - (g * dgate).sum(1, keepdims=True)), axis=1)
    np.testing.assert_allclose(O.gating_backward(p, idx, g, dgate, 1), closed, rtol=1e-11, atol=1e-15)
    ssel = np.take_along_axis(s, idx.astype(np.int64), 1)
    np.testing.assert_allclose(g, O.softmax(ssel), rtol=1e-13)


def test_mask_only_selects_which_weight_grads_exist():
    inp = _inputs(T=20, d=8, M=6, f=5, k=2, router_sigma=0.5)
    c = inp["cfg"]
    fwd = _fwd(inp)
    full = _bwd(inp, fwd)
    part = O.moe_backward(fwd, inp["dy"], inp["x"], inp["w_router"], inp["w_gate"], inp["w_up"], inp["w_down"],
                          c.renorm, wgrad_experts=[1, 4])
    assert sorted(part["d_w_gate"]) == [1, 4] and sorted(part["d_w_down"]) == [1, 4]
    assert np.array_equal(part["dx"], full["dx"]) and np.array_equal(part["d_w_router"], full["d_w_router"])
    for e in (1, 4):
        assert np.array_equal(part["d_w_up"][e], full["d_w_up"][e])
        one = O.expert_weight_grads(e, fwd, inp["dy"], inp["x"], inp["w_gate"][e], inp["w_up"][e], inp["w_down"][e])
        np.testing.assert_allclose(one[0], full["d_w_gate"][e], rtol=1e-13, atol=1e-18)
        np.testing.assert_allclose(one[2], full["d_w_down"][e], rtol=1e-13, atol=1e-18)
    # the gate gradient filled in one expert at a time equals the layer backward's, and with it the router gradient
    dgate = np.full(full["dgate"].shape, np.nan)
    for e in range(inp["cfg"].M):
        t_e, j_e, v = O.expert_gate_grads(e, fwd, inp["dy"], inp["x"], inp["w_gate"][e], inp["w_up"][e], inp["w_down"][e])
        dgate[t_e, j_e] = v
    np.testing.assert_allclose(dgate, full["dgate"], rtol=1e-12, atol=1e-18)
    dl = O.gating_backward(fwd["p"], fwd["idx"], fwd["gate"], dgate, inp["cfg"].renorm)
    np.testing.assert_allclose(dl.T @ inp["x"].astype(np.float64), full["d_w_router"], rtol=1e-10, atol=1e-16)


def test_forward_is_per_token():
    # evaluating a subset of tokens alone gives the same rows: large shapes can be checked on samples
    inp = _inputs(T=40, d=8, M=6, f=5, k=2, router_sigma=0.5, bias="normal", bias_scale=0.5)
    c = inp["cfg"]
    full = _fwd(inp)
    pick = np.array([3, 17, 39])
    sub = O.moe_forward(inp["x"][pick], inp["w_router"], inp["router_bias"], inp["w_gate"], inp["w_up"],
                        inp["w_down"], c.k, c.renorm)
    np.testing.assert_allclose(sub["y"], full["y"][pick], rtol=1e-13)
    assert np.array_equal(sub["idx"], full["idx"][pick])


@pytest.mark.parametrize("renorm", [0, 1])
def test_relabelling_the_experts_changes_nothing_but_the_labels(renorm):
    # Eq. 2 sums over a set of experts: renaming them (router rows, bias and weights together) must leave y and dx
    # alone and carry every per-expert result to its new name.  Catches an index used for the wrong tensor.
    inp = _inputs(T=50, d=8, M=7, f=6, k=3, renorm=renorm, router_sigma=0.7, bias="normal", bias_scale=0.3)
    c = inp["cfg"]
    fwd = _fwd(inp)
    bwd = _bwd(inp, fwd)
    rng = np.random.default_rng(5)
    new_of_old = rng.permutation(c.M)              # expert e is renamed new_of_old[e]
    old_of_new = np.argsort(new_of_old)
    x, dy = inp["x"], inp["dy"]
    wr, bias = inp["w_router"][old_of_new], inp["router_bias"][old_of_new]
    wg, wu, wd = inp["w_gate"][old_of_new], inp["w_up"][old_of_new], inp["w_down"][old_of_new]
    f2 = O.moe_forward(x, wr, bias, wg, wu, wd, c.k, c.renorm, keep=True)
    b2 = O.moe_backward(f2, dy, x, wr, wg, wu, wd, c.renorm)
    assert np.array_equal(f2["idx"], new_of_old[fwd["idx"]])
    np.testing.assert_allclose(f2["gate"], fwd["gate"], rtol=1e-13)
    np.testing.assert_allclose(f2["y"], fwd["y"], rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(b2["dx"], bwd["dx"], rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(b2["d_w_router"][new_of_old], bwd["d_w_router"], rtol=1e-11, atol=1e-14)
    assert np.array_equal(f2["count"][new_of_old], fwd["count"])
    for e in range(c.M):
        np.testing.assert_allclose(b2["d_w_gate"][int(new_of_old[e])], bwd["d_w_gate"][e], rtol=1e-11, atol=1e-14)
        np.testing.assert_allclose(b2["d_w_down"][int(new_of_old[e])], bwd["d_w_down"][e], rtol=1e-11, atol=1e-14)

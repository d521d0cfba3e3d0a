"""Pins for the oracle's router auxiliary losses (Sec. 3.3 "Training Losses"; coefficients App. B):
closed forms, a library autograd pass written from the definitions, and finite differences."""
import math

import numpy as np
import torch

from oracle import spes_oracle as O


def _case(T=37, M=8, k=2, seed=3, scale=1.5):
    rng = np.random.default_rng(seed)
    s = rng.normal(size=(T, M)) * scale
    return s, O.top_k(s, k)


def test_uniform_scores_closed_form():
    """All-equal scores: P_e = 1/M, so L_lb = sum_e f_e = 1 whatever the routing; lse = c + ln M."""
    T, M, k = 12, 8, 2
    s = np.full((T, M), 0.7)
    idx = np.stack([np.arange(T) % M, (np.arange(T) + 3) % M], axis=1).astype(np.int32)
    lb, z, f, P = O.router_aux_losses(s, idx)
    assert abs(lb - 1.0) < 1e-14
    assert abs(z - (0.7 + math.log(M)) ** 2) < 1e-13
    assert abs(f.sum() - 1.0) < 1e-15 and np.allclose(P, 1.0 / M)


def test_collapsed_routing_closed_form():
    """Every token sends all its probability mass and both its choices' worth of traffic to one expert:
    one-hot p (in the limit) and f = (1/k, ..) -> L_lb -> M * f_0 * 1."""
    T, M, k = 16, 4, 2
    s = np.zeros((T, M)); s[:, 0] = 60.0; s[:, 1] = 1.0           # top-2 = experts 0 and 1
    idx = O.top_k(s, k)
    lb, z, f, P = O.router_aux_losses(s, idx)
    assert np.allclose(f, [0.5, 0.5, 0, 0])
    assert abs(lb - M * 0.5) < 1e-12                              # P_0 = 1 to rounding, P_1 ~ e^-59
    assert abs(z - 60.0 ** 2) < 1e-9


def test_losses_match_autograd_definitions():
    s, idx = _case()
    T, M = s.shape
    k = idx.shape[1]
    lb, z, f, P = O.router_aux_losses(s, idx)
    ts = torch.tensor(s, dtype=torch.float64, requires_grad=True)
    onehot = torch.zeros(T, M, dtype=torch.float64)
    onehot.scatter_add_(1, torch.tensor(idx, dtype=torch.int64), torch.ones(T, k, dtype=torch.float64))
    tf = onehot.sum(0) / (T * k)
    tlb = M * (tf * torch.softmax(ts, dim=1).mean(0)).sum()
    tz = (torch.logsumexp(ts, dim=1) ** 2).mean()
    assert abs(lb - tlb.item()) < 1e-13 and abs(z - tz.item()) < 1e-12
    lb_coef, z_coef, gs = 0.01, 0.001, 3.0
    (gs * (lb_coef * tlb + z_coef * tz)).backward()
    got = O.router_aux_dlogits(s, idx, lb_coef, z_coef, gs)
    np.testing.assert_allclose(got, ts.grad.numpy(), rtol=1e-11, atol=1e-16)


def test_dlogits_finite_differences_and_row_sums():
    s, idx = _case(T=9, M=5, k=2, seed=11)
    lb_coef, z_coef = 0.3, 0.2
    g = O.router_aux_dlogits(s, idx, lb_coef, z_coef)
    eps = 1e-6
    for (t, e) in [(0, 0), (3, 4), (8, 2)]:
        sp, sm = s.copy(), s.copy()
        sp[t, e] += eps; sm[t, e] -= eps
        lp = O.router_aux_losses(sp, idx); lm = O.router_aux_losses(sm, idx)   # idx held fixed: counts carry no gradient
        fd = (lb_coef * (lp[0] - lm[0]) + z_coef * (lp[1] - lm[1])) / (2 * eps)
        assert abs(fd - g[t, e]) < 1e-8
    # the load-balancing part is a softmax-Jacobian product (rows sum to zero); the z part sums to 2 z lse / T
    only_lb = O.router_aux_dlogits(s, idx, 1.0, 0.0)
    assert np.abs(only_lb.sum(axis=1)).max() < 1e-15
    only_z = O.router_aux_dlogits(s, idx, 0.0, 1.0)
    lse = np.log(np.exp(s).sum(axis=1))
    np.testing.assert_allclose(only_z.sum(axis=1), 2 * lse / s.shape[0], rtol=1e-12)


def test_extra_dlogits_reaches_router_and_input():
    """moe_backward adds the auxiliary gradient to dlogits: d_w_router and dx move by extra^T x and extra W_r."""
    rng = np.random.default_rng(5)
    T, d, M, f, k = 20, 6, 4, 5, 2
    x = rng.normal(size=(T, d)); wr = rng.normal(size=(M, d)) * 0.3
    wg = rng.normal(size=(M, f, d)) * 0.3; wu = rng.normal(size=(M, f, d)) * 0.3; wd = rng.normal(size=(M, d, f)) * 0.3
    dy = rng.normal(size=(T, d))
    fwd = O.moe_forward(x, wr, None, wg, wu, wd, k, 0)
    extra = O.router_aux_dlogits(fwd["logits"], fwd["idx"], 0.01, 0.001)
    b0 = O.moe_backward(fwd, dy, x, wr, wg, wu, wd, 0)
    b1 = O.moe_backward(fwd, dy, x, wr, wg, wu, wd, 0, extra_dlogits=extra)
    np.testing.assert_allclose(b1["d_w_router"] - b0["d_w_router"], extra.T @ x, rtol=1e-9, atol=1e-15)
    np.testing.assert_allclose(b1["dx"] - b0["dx"], extra @ wr, rtol=1e-9, atol=1e-15)
    for e in range(M):
        np.testing.assert_array_equal(b1["d_w_gate"][e], b0["d_w_gate"][e])

"""Pins for the oracle's AdamW step: the library optimizer, closed forms of the first step, and the mask."""
import numpy as np
import torch

from oracle import spes_oracle as O

HYPER = dict(lr=5e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)     # App. B, Table A1 (1B / 2B column)


def test_matches_library_adamw_over_several_steps():
    rng = np.random.default_rng(0)
    w0 = rng.normal(size=(7, 5)) * 0.02
    p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=HYPER["lr"], betas=(HYPER["beta1"], HYPER["beta2"]), eps=HYPER["eps"],
                            weight_decay=HYPER["weight_decay"])
    w, m, v = w0.copy(), np.zeros_like(w0), np.zeros_like(w0)
    for step in range(1, 6):
        g = rng.normal(size=w0.shape) * (0.1 if step % 2 else 3.0)
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        w, m, v = O.adamw_step(w, m, v, g, step=step, **HYPER)
        np.testing.assert_allclose(w, p.detach().numpy(), rtol=1e-12, atol=1e-18)
    st = opt.state[p]
    np.testing.assert_allclose(m, st["exp_avg"].numpy(), rtol=1e-12)
    np.testing.assert_allclose(v, st["exp_avg_sq"].numpy(), rtol=1e-12)


def test_first_step_closed_form():
    """From zero moments the bias corrections cancel: m_hat = g, v_hat = g^2, so the step is lr*(sign(g) + wd*w)
    up to eps; the moments are (1-beta) g and (1-beta2) g^2."""
    w = np.array([1.0, -2.0, 0.5]); g = np.array([0.3, -4.0, 1e-3])
    nw, nm, nv = O.adamw_step(w, np.zeros(3), np.zeros(3), g, step=1, **HYPER)
    want = w - HYPER["lr"] * (g / (np.abs(g) + HYPER["eps"]) + HYPER["weight_decay"] * w)
    np.testing.assert_allclose(nw, want, rtol=1e-14)
    np.testing.assert_allclose(nm, 0.1 * g, rtol=1e-14)
    np.testing.assert_allclose(nv, 0.05 * g * g, rtol=1e-13)


def test_zero_gradient_only_decays_and_grad_scale_is_linear():
    w = np.array([2.0, -1.0])
    nw, nm, nv = O.adamw_step(w, np.zeros(2), np.zeros(2), np.zeros(2), step=3, **HYPER)
    np.testing.assert_allclose(nw, w * (1 - HYPER["lr"] * HYPER["weight_decay"]), rtol=1e-15)
    assert not nm.any() and not nv.any()
    g = np.array([0.2, -0.7])
    a = O.adamw_step(w, np.ones(2) * 0.1, np.ones(2) * 0.2, g, step=4, grad_scale=0.25, **HYPER)
    b = O.adamw_step(w, np.ones(2) * 0.1, np.ones(2) * 0.2, g * 0.25, step=4, **HYPER)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, rtol=1e-15)


def test_mask_leaves_frozen_experts_alone():
    rng = np.random.default_rng(1)
    M, n = 6, 4
    param = rng.normal(size=(M, n)); trainable = [1, 4]
    master = param[trainable].copy(); m = rng.normal(size=(2, n)) * 0.01; v = rng.random(size=(2, n)) * 0.01
    grad = rng.normal(size=(2, n))
    np_, nmaster, nm, nv = O.masked_adamw(param, trainable, master, m, v, grad, step=2, **HYPER)
    for e in range(M):
        if e not in trainable:
            np.testing.assert_array_equal(np_[e], param[e])
    for s, e in enumerate(trainable):
        w1, m1, v1 = O.adamw_step(master[s], m[s], v[s], grad[s], step=2, **HYPER)
        np.testing.assert_array_equal(np_[e], w1)
        np.testing.assert_array_equal(nmaster[s], w1)
        np.testing.assert_array_equal(nm[s], m1)
        np.testing.assert_array_equal(nv[s], v1)

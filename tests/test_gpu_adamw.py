"""AdamW on the trainable subset: device kernel against the fp64 oracle through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2602_11543_amd as S
from harness import TOL, rel_err
from oracle import spes_oracle as O
from spes_workloads import bf16_round

pytestmark = pytest.mark.gpu

HYPER = dict(lr=5e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)     # App. B, Table A1


def _run(device, M, elems, mask, dtype, steps, with_master=True, seed=0, grad_scale=1.0):
    rng = np.random.default_rng(seed)
    trainable = [int(e) for e in np.nonzero(mask)[0]]
    n = len(trainable)
    p0 = rng.normal(size=(M, elems)) * 0.02
    p0 = bf16_round(p0) if dtype == "bf16" else p0.astype(np.float32).astype(np.float64)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    param = torch.from_numpy(p0).to(tdt).to(device)
    master0 = p0[trainable].copy()
    master = torch.from_numpy(master0).float().to(device) if with_master else None
    m = torch.zeros(n, elems, dtype=torch.float32, device=device)
    v = torch.zeros(n, elems, dtype=torch.float32, device=device)
    o_param, o_master, o_m, o_v = p0.copy(), master0.copy(), np.zeros((n, elems)), np.zeros((n, elems))
    for step in range(1, steps + 1):
        g = (rng.normal(size=(n, elems)) * (3.0 if step == 2 else 0.05)).astype(np.float32)
        grad = torch.from_numpy(g).to(device)
        S.spes_masked_adamw(M, elems, S.SPES_BF16 if dtype == "bf16" else S.SPES_F32, param, mask, master, m, v, grad,
                            step=step, grad_scale=grad_scale, **HYPER)
        o_param, o_master, o_m, o_v = O.masked_adamw(o_param, trainable, o_master, o_m, o_v, g.astype(np.float64), step=step,
                                                     grad_scale=grad_scale, **HYPER)
    torch.cuda.synchronize()
    return dict(param=param, master=master, m=m, v=v, p0=p0, trainable=trainable,
                o_param=o_param, o_master=o_master, o_m=o_m, o_v=o_v)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_parity_over_steps(device, dtype):
    M, elems = 8, 8 * 1027                      # several blocks and a ragged tail
    mask = np.array([0, 1, 0, 0, 1, 1, 0, 0], dtype=np.uint8)
    r = _run(device, M, elems, mask, dtype, steps=4, grad_scale=0.5)
    tol = TOL["f32"]                             # all arithmetic is fp32 whatever the storage type
    assert rel_err(r["m"].cpu().numpy(), r["o_m"]) < tol
    assert rel_err(r["v"].cpu().numpy(), r["o_v"]) < tol
    assert rel_err(r["master"].cpu().numpy(), r["o_master"]) < tol
    got = r["param"].float().cpu().numpy().astype(np.float64)
    for s, e in enumerate(r["trainable"]):
        dev_master = r["master"][s].cpu().numpy().astype(np.float64)
        want = bf16_round(dev_master) if dtype == "bf16" else dev_master
        assert np.array_equal(got[e], want), "the store must hold the rounded fp32 weight"
    for e in range(M):
        if not mask[e]:
            assert np.array_equal(got[e], r["p0"][e]), "frozen expert changed"


def test_f32_store_is_its_own_master(device):
    M, elems = 3, 8 * 130
    mask = np.array([1, 0, 1], dtype=np.uint8)
    r = _run(device, M, elems, mask, "f32", steps=3, with_master=False)
    got = r["param"].cpu().numpy().astype(np.float64)
    assert rel_err(got[r["trainable"]], r["o_master"]) < TOL["f32"]
    assert np.array_equal(got[1], r["p0"][1])


def test_more_slots_than_one_launch_and_no_trainable(device):
    M, elems = 70, 64
    r = _run(device, M, elems, np.ones(M, dtype=np.uint8), "bf16", steps=2)
    assert rel_err(r["master"].cpu().numpy(), r["o_master"]) < TOL["f32"]
    assert rel_err(r["m"].cpu().numpy(), r["o_m"]) < TOL["f32"]
    # nothing trainable: a no-op that needs no state buffers
    param = torch.ones(4, 64, dtype=torch.bfloat16, device=device)
    S.spes_masked_adamw(4, 64, S.SPES_BF16, param, np.zeros(4, dtype=np.uint8), None, None, None, None, step=1, **HYPER)
    torch.cuda.synchronize()
    assert bool((param == 1).all())


def test_argument_errors(device):
    t = torch.zeros(2, 64, dtype=torch.float32, device=device)
    p = torch.zeros(2, 64, dtype=torch.bfloat16, device=device)
    mask = np.array([1, 1], dtype=np.uint8)
    with pytest.raises(S.SpesError):
        S.spes_masked_adamw(2, 64, S.SPES_BF16, p, mask, None, t, t, t, step=1, **HYPER)      # bf16 store needs fp32 weights
    with pytest.raises(S.SpesError):
        S.spes_masked_adamw(2, 64, S.SPES_BF16, p, mask, t, t, t, t, step=0, **HYPER)         # steps count from 1
    with pytest.raises(S.SpesError):
        S.spes_masked_adamw(2, 60, S.SPES_BF16, p, mask, t, t, t, t, step=1, **HYPER)         # elems not a multiple of 8


def test_full_size_matrix_sampled(device):
    """One cfg2-shaped matrix (16 trainable of 64 experts, 2048 x 1024 each): sampled elements against the oracle."""
    M, elems, n = 64, 2048 * 1024, 16
    rng = np.random.default_rng(7)
    mask = np.zeros(M, dtype=np.uint8); mask[rng.choice(M, n, replace=False)] = 1
    trainable = [int(e) for e in np.nonzero(mask)[0]]
    gen = torch.Generator(device="cpu").manual_seed(3)
    p0 = (torch.randn(M, elems, generator=gen) * 0.02).to(torch.bfloat16)
    param = p0.to(device)
    master = p0[trainable].float().to(device)
    m = (torch.randn(n, elems, generator=gen) * 0.01).to(device)
    v = (torch.rand(n, elems, generator=gen) * 1e-3).to(device)
    grad = (torch.randn(n, elems, generator=gen) * 0.1).to(device)
    m0, v0, w0, g0 = m.cpu().numpy(), v.cpu().numpy(), master.cpu().numpy(), grad.cpu().numpy()
    S.spes_masked_adamw(M, elems, S.SPES_BF16, param, mask, master, m, v, grad, step=7, **HYPER)
    torch.cuda.synchronize()
    cols = np.concatenate([rng.choice(elems, 4096, replace=False), [0, 1, elems - 2, elems - 1]])
    ow, om, ov = O.adamw_step(w0[:, cols], m0[:, cols], v0[:, cols], g0[:, cols], step=7, **HYPER)
    assert rel_err(master.cpu().numpy()[:, cols], ow) < TOL["f32"]
    assert rel_err(m.cpu().numpy()[:, cols], om) < TOL["f32"]
    assert rel_err(v.cpu().numpy()[:, cols], ov) < TOL["f32"]
    frozen = [e for e in range(M) if not mask[e]]
    assert torch.equal(param[frozen].cpu(), p0[frozen])
    assert torch.equal(param[trainable].cpu(), master.cpu().to(torch.bfloat16))

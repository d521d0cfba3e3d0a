"""Upcycling initialiser and pack / unpack of trained experts on the device against the oracle."""
import numpy as np
import pytest
import torch

import paper_2602_11543_amd as S
from harness import TOL, rel_err
from oracle import spes_oracle as O
from spes_workloads import bf16_round

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_upcycle_small_every_element(device, dtype):
    M, elems, frac, sigma, seed, sid = 5, 8 * 257, 0.5, 0.02, 20260211, 3
    rng = np.random.default_rng(0)
    dense = rng.normal(size=elems) * 0.02
    dense = bf16_round(dense) if dtype == "bf16" else dense.astype(np.float32).astype(np.float64)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    d_dense = torch.from_numpy(dense).to(tdt).to(device)
    out = torch.empty(M, elems, dtype=tdt, device=device)
    S.spes_upcycle_init(M, elems, S.SPES_BF16 if dtype == "bf16" else S.SPES_F32, d_dense, frac, sigma, seed, sid, out)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    want = O.upcycle_init(dense, M, frac, sigma, seed, sid)
    if dtype == "f32":
        assert rel_err(got, want) < TOL["f32"]
        assert np.array_equal(got != dense[None, :], want != dense[None, :])      # the same elements were selected
    else:
        want_r = bf16_round(want)
        # the noise is computed in fp32 on the device and fp64 here: a sum that lands within rounding distance of a
        # bf16 tie may round the other way; everything else must be identical
        diff = got != want_r
        assert diff.mean() < 5e-3, diff.mean()
        assert np.abs(got - want_r)[diff].max() <= np.abs(want_r[diff]).max() * 2.0 ** -7
        assert rel_err(got, want) < TOL["bf16"]
    # unselected elements are exact copies
    same = want == dense[None, :]
    assert np.array_equal(got[same], np.broadcast_to(dense, got.shape)[same])


def test_upcycle_full_size_sampled_and_moments(device):
    """The upcycled workload's gate projection: 32 experts of 4864 x 3584 from one dense matrix."""
    M, elems, frac, sigma, seed, sid = 32, 4864 * 3584, 0.5, 0.02, 7, 1
    gen = torch.Generator(device="cpu").manual_seed(5)
    dense = (torch.randn(elems, generator=gen) * 0.02).to(torch.bfloat16)
    d_dense = dense.to(device)
    out = torch.empty(M, elems, dtype=torch.bfloat16, device=device)
    S.spes_upcycle_init(M, elems, S.SPES_BF16, d_dense, frac, sigma, seed, sid, out)
    torch.cuda.synchronize()
    delta = out.float() - d_dense.float()[None, :]
    changed = delta != 0
    share = float(changed.float().mean())
    assert abs(share - 0.5) < 2e-3, share              # (a selected element whose noise rounds away counts as unchanged)
    std = float(delta[changed].std())
    assert abs(std - sigma) < 2e-4, std
    assert abs(float(delta[changed].mean())) < 1e-4
    # sampled groups against the oracle's draws
    rng = np.random.default_rng(1)
    dn = dense.float().numpy().astype(np.float64)
    thr = 128
    bad = 0
    checked = 0
    for e, g in zip(rng.integers(0, M, 1500), rng.integers(0, elems // 4, 1500)):
        sel, z = O.upcycle_draws((int(e) * elems) // 4 + int(g), seed, sid)
        got = out[int(e), 4 * int(g):4 * int(g) + 4].float().cpu().numpy().astype(np.float64)
        for j in range(4):
            want = dn[4 * g + j] + (sigma * z[j] if sel[j] < thr else 0.0)
            wr = float(bf16_round(np.array([want]))[0])
            checked += 1
            if got[j] != wr:
                bad += 1
                assert abs(got[j] - wr) <= abs(wr) * 2.0 ** -7
    assert bad <= checked * 5e-3, (bad, checked)


def test_upcycle_argument_errors(device):
    d = torch.zeros(64, dtype=torch.bfloat16, device=device)
    o = torch.zeros(2, 64, dtype=torch.bfloat16, device=device)
    with pytest.raises(S.SpesError):
        S.spes_upcycle_init(2, 64, S.SPES_BF16, d, 1.5, 0.02, 1, 0, o)
    with pytest.raises(S.SpesError):
        S.spes_upcycle_init(2, 60, S.SPES_BF16, d, 0.5, 0.02, 1, 0, o)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_pack_unpack(device, dtype):
    M, elems = 70, 8 * 37
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    sd = S.SPES_BF16 if dtype == "bf16" else S.SPES_F32
    gen = torch.Generator(device="cpu").manual_seed(2)
    store = torch.randn(M, elems, generator=gen).to(tdt).to(device)
    mask = np.ones(M, dtype=np.uint8); mask[[0, 5, 69]] = 0               # 67 slots: more than one launch
    tr = [int(e) for e in np.nonzero(mask)[0]]
    packed = torch.zeros(len(tr), elems, dtype=tdt, device=device)
    S.spes_expert_pack(M, elems, sd, store, mask, packed, 0)
    torch.cuda.synchronize()
    assert torch.equal(packed, store[tr])
    new = torch.randn(len(tr), elems, generator=gen).to(tdt).to(device)
    before = store.clone()
    S.spes_expert_pack(M, elems, sd, store, mask, new, 1)
    torch.cuda.synchronize()
    assert torch.equal(store[tr], new)
    assert torch.equal(store[[0, 5, 69]], before[[0, 5, 69]])
    # nothing trainable: no-op without a buffer
    S.spes_expert_pack(M, elems, sd, store, np.zeros(M, dtype=np.uint8), None, 0)

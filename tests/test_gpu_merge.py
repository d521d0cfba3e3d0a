"""GPU parity of spes_expert_merge / spes_expert_warmup_merge against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2602_11543_amd as S
from oracle import spes_oracle as O
from spes_workloads import bf16_round, merge_inputs

from harness import TOL, rel_err, storage_ulp_excess, to_dev

pytestmark = pytest.mark.gpu


def _host(t):
    return t.float().cpu().numpy() if t.dtype == torch.bfloat16 else t.cpu().numpy()


def _run_merge(mi, dtype, device):
    M, E = mi["base"].shape
    dst = to_dev(mi["base"], dtype, device)
    stores = [to_dev(s, dtype, device) for s in mi["stores"]]
    cnt = torch.full((M,), -7, dtype=torch.int32, device=device)
    S.spes_expert_merge(M, E, S.SPES_F32 if dtype == "f32" else S.SPES_BF16, stores, mi["slot"], mi["node_weight"], dst, cnt)
    torch.cuda.synchronize()
    return _host(dst), cnt.cpu().numpy()


def _round(a, dtype):
    return bf16_round(a.astype(np.float32)).astype(np.float64) if dtype == "bf16" else a


@pytest.mark.parametrize("dtype,M,E,nodes,per,weighted", [
    ("f32", 8, 3 * 256 * 512, 4, None, False),        # the small configuration: 4 full copies, uniform (FedAvg)
    ("bf16", 64, 4096 + 8, 16, 16, True),              # 16 nodes x 16 experts, weighted, ragged vector tail
    ("bf16", 64, 2048, 16, 16, False),
    ("f32", 40, 1000, 7, 5, True),
])
def test_sync_merge_parity(dtype, M, E, nodes, per, weighted, device):
    print(f"[case] merge {dtype} M={M} E={E} nodes={nodes}", flush=True)
    mi = merge_inputs(M, E, nodes, per, dtype, seed=77 + M, weighted=weighted, need_zero_and_single=per is not None)
    got, cnt = _run_merge(mi, dtype, device)
    want, wcnt = O.sync_merge(mi["base"], mi["stores"], mi["slot"], mi["node_weight"])
    assert np.array_equal(cnt, wcnt)
    # element by element: one bf16 ulp from the rounded fp64 mean; in fp32 two ulps at the magnitude of the copies
    mag = np.abs(mi["base"]).astype(np.float32)
    for i, st in enumerate(mi["stores"]):
        for j in np.nonzero(mi["slot"][i] >= 0)[0]:
            mag[j] = np.maximum(mag[j], np.abs(st[mi["slot"][i, j]]))
    assert storage_ulp_excess(got, want, mag, dtype) <= 0
    untouched = np.nonzero(wcnt == 0)[0]
    single = np.nonzero(wcnt == 1)[0]
    for j in untouched:
        assert np.array_equal(got[j], mi["base"][j])                 # no trainer: previous value kept
    for j in single:                                                   # one trainer: direct, bit-exact assignment
        i = int(np.nonzero(mi["slot"][:, j] >= 0)[0][0])
        assert np.array_equal(got[j], mi["stores"][i][mi["slot"][i, j]])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sync_merge_identical_copies_is_identity(dtype, device):
    mi = merge_inputs(12, 520, 9, None, dtype, seed=5, noise=0.0, weighted=True)
    got, cnt = _run_merge(mi, dtype, device)
    assert np.array_equal(got, mi["base"]) and cnt.tolist() == [9] * 12


def test_sync_merge_weight_scale_invariance_and_errors(device):
    mi = merge_inputs(10, 256, 6, 4, "f32", seed=8, weighted=True)
    a, _ = _run_merge(mi, "f32", device)
    mi2 = dict(mi); mi2["node_weight"] = (mi["node_weight"] * 4.0).astype(np.float32)   # power of two: exact
    b, _ = _run_merge(mi2, "f32", device)
    assert np.array_equal(a, b)
    dst = to_dev(mi["base"], "f32", device)
    stores = [to_dev(s, "f32", device) for s in mi["stores"]]
    with pytest.raises(S.SpesError, match="unsupported"):
        S.spes_expert_merge(10, 252, S.SPES_F32, stores, mi["slot"], None, dst, None)
    with pytest.raises(S.SpesError, match="invalid"):
        S.spes_expert_merge(10, 256, S.SPES_F32, stores, mi["slot"], np.zeros(6, np.float32), dst, None)


def _structured_experts(M, E, dtype, seed):
    """Experts in loose clusters so that similarities are well separated."""
    rng = np.random.default_rng(seed)
    centres = rng.standard_normal((4, E))
    w = np.stack([centres[j % 4] * (1.0 + 0.1 * (j // 4)) + (0.15 + 0.05 * j) * rng.standard_normal(E) for j in range(M)]) * 0.02
    w = w.astype(np.float32)
    return bf16_round(w) if dtype == "bf16" else w


@pytest.mark.parametrize("dtype,M,E,K,alpha", [("f32", 8, 4096, 4, 0.1), ("bf16", 64, 8200, 4, 0.1), ("bf16", 16, 3000 * 8, 3, 1.0),
                                               ("f32", 6, 512, 5, 1.0), ("f32", 8, 1024, 4, 0.0),
                                               # several column runs per XCD with a ragged last run, K not a multiple of
                                               # the four peers requested at a time; K = M - 1 with whole XCD turns empty
                                               ("bf16", 24, 8 * (2048 * 8 + 5), 7, 0.3), ("f32", 12, 8 * (128 * 9 + 1), 11, 0.5)])
def test_warmup_merge_parity(dtype, M, E, K, alpha, device):
    print(f"[case] warmup {dtype} M={M} E={E} K={K} alpha={alpha}", flush=True)
    dt = S.SPES_F32 if dtype == "f32" else S.SPES_BF16
    w_in = _structured_experts(M, E, dtype, 1)
    others = [_structured_experts(M, E2, dtype, 2 + i) for i, E2 in enumerate((E, 264))]
    mats = [w_in] + others
    d_src = [to_dev(m, dtype, device) for m in mats]
    d_dst = [torch.zeros_like(t) for t in d_src]
    sim = torch.zeros(M, M, dtype=torch.float32, device=device)
    nbr = torch.zeros(M, K, dtype=torch.int32, device=device)
    scratch = torch.empty(S.spes_warmup_scratch_bytes(M, E), dtype=torch.uint8, device=device)
    S.spes_expert_warmup_merge(M, dt, K, alpha, d_src[0], E, d_src, d_dst, [m.shape[1] for m in mats], sim, nbr, scratch)
    torch.cuda.synchronize()
    A = O.cosine_similarity(w_in)
    assert np.abs(sim.cpu().numpy() - A).max() <= 2e-5
    want_nbr = O.top_K_neighbours(A, K)
    got_nbr = nbr.cpu().numpy()
    # the peer set is decided in fp32 on the GPU: it must be the oracle's wherever the oracle's choice is clear-cut
    for j in range(M):
        row = A[j].copy(); row[j] = -np.inf
        srt = np.sort(row)[::-1]
        clear = (srt[K - 1] - srt[K]) > 1e-4 if K < M - 1 else True
        assert j not in got_nbr[j] and len(set(got_nbr[j].tolist())) == K
        if clear:
            assert set(got_nbr[j].tolist()) == set(want_nbr[j].tolist())
        assert np.all(row[got_nbr[j]] >= srt[K - 1] - 1e-4)
    tol = TOL[dtype]
    for m, t in zip(mats, d_dst):
        want = O.warmup_merge(m, got_nbr, alpha)
        mag = np.abs(m).astype(np.float32)
        mag = np.maximum(mag, np.abs(m[got_nbr]).max(axis=1))          # an expert's own row and its K peers' rows
        assert storage_ulp_excess(_host(t), want, mag, dtype, f32_ulps=K + 2.0) <= 0
        if alpha == 0.0:
            assert np.array_equal(_host(t), m)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_warmup_merge_with_a_zero_norm_expert(dtype, device):
    """An all-zero input projection makes Eq. 5 a 0/0: the pair gets similarity 0, peers stay valid experts."""
    M, E, K, alpha = 12, 2048, 4, 0.3
    dt = S.SPES_F32 if dtype == "f32" else S.SPES_BF16
    w_in = _structured_experts(M, E, dtype, 21)
    w_in[5] = 0.0
    other = _structured_experts(M, 520, dtype, 22)
    mats = [w_in, other]
    d_src = [to_dev(m, dtype, device) for m in mats]
    d_dst = [torch.zeros_like(t) for t in d_src]
    sim = torch.full((M, M), float("nan"), dtype=torch.float32, device=device)
    nbr = torch.full((M, K), -1, dtype=torch.int32, device=device)
    scratch = torch.empty(S.spes_warmup_scratch_bytes(M, E), dtype=torch.uint8, device=device)
    S.spes_expert_warmup_merge(M, dt, K, alpha, d_src[0], E, d_src, d_dst, [m.shape[1] for m in mats], sim, nbr, scratch)
    torch.cuda.synchronize()
    A = O.cosine_similarity(w_in)
    got_sim, got_nbr = sim.cpu().numpy(), nbr.cpu().numpy()
    assert np.all(got_sim[5] == 0.0) and np.all(got_sim[:, 5] == 0.0)
    assert np.abs(got_sim - A).max() <= 2e-5
    want_nbr = O.top_K_neighbours(A, K)
    assert got_nbr[5].tolist() == want_nbr[5].tolist() == [0, 1, 2, 3]          # all equal: the lowest ids
    for j in range(M):
        assert j not in got_nbr[j] and len(set(got_nbr[j].tolist())) == K and got_nbr[j].min() >= 0 and got_nbr[j].max() < M
    for m, t in zip(mats, d_dst):
        want = O.warmup_merge(m, got_nbr, alpha)
        mag = np.maximum(np.abs(m).astype(np.float32), np.abs(m[got_nbr]).max(axis=1))
        assert storage_ulp_excess(_host(t), want, mag, dtype, f32_ulps=K + 2.0) <= 0

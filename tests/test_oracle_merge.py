"""Pins for the oracle's synchronisation and expert-merging warm-up (CPU only)."""
import numpy as np
import pytest
from scipy.spatial.distance import cosine as sp_cosine_distance

from oracle import spes_oracle as O
from spes_workloads import merge_inputs


def test_sync_identical_copies_is_identity():
    mi = merge_inputs(M=5, elems=40, n_nodes=4, experts_per_node=None, dtype="f32", seed=3, noise=0.0)
    dst, cnt = O.sync_merge(mi["base"], mi["stores"], mi["slot"], mi["node_weight"])
    np.testing.assert_allclose(dst, mi["base"], rtol=1e-15)
    assert cnt.tolist() == [4] * 5


def test_sync_single_owner_is_direct_assignment():
    # a disjoint partition: expert j is owned by node j % 3 (Eq. 4, second component)
    rng = np.random.default_rng(0)
    M, E, N = 7, 11, 3
    base = rng.standard_normal((M, E))
    slot = np.full((N, M), -1, dtype=np.int32)
    stores = []
    for i in range(N):
        own = [j for j in range(M) if j % N == i]
        slot[i, own] = np.arange(len(own))
        stores.append(rng.standard_normal((len(own), E)))
    dst, cnt = O.sync_merge(base, stores, slot, rng.random(N) + 0.5)
    assert cnt.tolist() == [1] * M
    for j in range(M):
        np.testing.assert_allclose(dst[j], stores[j % N][slot[j % N, j]], rtol=5e-16)   # w*phi/w: one fp64 rounding


def test_sync_all_nodes_uniform_is_fedavg_mean():
    mi = merge_inputs(M=4, elems=33, n_nodes=6, experts_per_node=None, dtype="f32", seed=4, weighted=False)
    dst, _ = O.sync_merge(mi["base"], mi["stores"], mi["slot"], None)
    np.testing.assert_allclose(dst, np.mean(np.stack(mi["stores"]).astype(np.float64), axis=0), rtol=1e-14)


def test_sync_bruteforce_weighted_untrained_and_scaling():
    mi = merge_inputs(M=12, elems=9, n_nodes=5, experts_per_node=3, dtype="bf16", seed=9, need_zero_and_single=True)
    dst, cnt = O.sync_merge(mi["base"], mi["stores"], mi["slot"], mi["node_weight"])
    assert np.array_equal(cnt, (mi["slot"] >= 0).sum(0)) and cnt.sum() == 15
    assert (cnt == 0).any() and (cnt == 1).any()
    for j in range(12):
        for c in range(9):
            num = den = 0.0
            for i in range(5):
                s = mi["slot"][i, j]
                if s >= 0:
                    num += float(mi["node_weight"][i]) * float(mi["stores"][i][s, c]); den += float(mi["node_weight"][i])
            want = num / den if den else float(mi["base"][j, c])
            assert abs(dst[j, c] - want) <= 1e-15 * max(1.0, abs(want))
    dst2, _ = O.sync_merge(mi["base"], mi["stores"], mi["slot"], 7.5 * mi["node_weight"].astype(np.float64))
    np.testing.assert_allclose(dst2, dst, rtol=1e-14)


def test_average_of_deltas_equals_average_of_copies():
    # Eq. 1 with an SGD outer step of size 1: theta + mean(theta_i - theta) = mean(theta_i)
    mi = merge_inputs(M=3, elems=21, n_nodes=4, experts_per_node=None, dtype="f32", seed=5, weighted=False)
    base = mi["base"].astype(np.float64)
    deltas = np.mean([s.astype(np.float64) - base for s in mi["stores"]], axis=0)
    dst, _ = O.sync_merge(mi["base"], mi["stores"], mi["slot"], None)
    np.testing.assert_allclose(dst, base + deltas, rtol=1e-12, atol=1e-16)


# ---------------------------------------------------------------- warm-up merge

def test_cosine_similarity_properties_and_library():
    rng = np.random.default_rng(1)
    w = rng.standard_normal((6, 50))
    A = O.cosine_similarity(w)
    np.testing.assert_allclose(A, A.T, rtol=1e-14)
    np.testing.assert_allclose(np.diag(A), 1.0, rtol=1e-14)
    assert np.all(np.abs(A) <= 1 + 1e-14)
    np.testing.assert_allclose(O.cosine_similarity(w * rng.uniform(0.1, 9.0, (6, 1))), A, rtol=1e-12)
    for j in range(6):
        for k in range(6):
            if j != k:
                assert abs(A[j, k] - (1.0 - sp_cosine_distance(w[j], w[k]))) < 1e-13
    w3 = rng.standard_normal((4, 5, 7))                     # a [M,f,d] projection is flattened
    np.testing.assert_allclose(O.cosine_similarity(w3), O.cosine_similarity(w3.reshape(4, -1)))


def test_zero_norm_projection_has_similarity_zero_and_is_never_preferred():
    # Eq. 5 is 0/0 for an all-zero input projection; the reading: similarity 0 for every pair it is part of
    rng = np.random.default_rng(11)
    w = rng.standard_normal((6, 40))
    ref = O.cosine_similarity(w)
    w[3] = 0.0
    A = O.cosine_similarity(w)
    assert np.all(np.isfinite(A))
    assert np.all(A[3] == 0.0) and np.all(A[:, 3] == 0.0)
    keep = [0, 1, 2, 4, 5]
    np.testing.assert_array_equal(A[np.ix_(keep, keep)], ref[np.ix_(keep, keep)])       # the other pairs are untouched
    nbr = O.top_K_neighbours(A, 2)
    assert nbr[3].tolist() == [0, 1]                                                     # all ties: lowest ids, never itself
    for j in keep:                                                                       # 0 ranks between the positive and the negative ones
        cand = sorted((k for k in range(6) if k != j), key=lambda k: (-A[j, k], k))
        assert nbr[j].tolist() == cand[:2] and j not in nbr[j]
    phi = rng.standard_normal((6, 12)); phi[3] = 0.0
    out = O.warmup_merge(phi, nbr, 0.5)
    np.testing.assert_allclose(out[3], 0.25 * (phi[0] + phi[1]), rtol=1e-14)             # Eq. 6 on the zero expert


def test_top_K_neighbours_bruteforce():
    rng = np.random.default_rng(2)
    A = rng.standard_normal((9, 9)); A = (A + A.T) / 2
    A[2, 5] = A[2, 7] = 10.0                                # tie: lower index first
    nbr = O.top_K_neighbours(A, 4)
    for j in range(9):
        cand = sorted((k for k in range(9) if k != j), key=lambda k: (-A[j, k], k))
        assert nbr[j].tolist() == cand[:4]
        assert j not in nbr[j]
    assert nbr[2, :2].tolist() == [5, 7]


def test_warmup_merge_invariants():
    rng = np.random.default_rng(3)
    M, E, K = 7, 30, 3
    phi = rng.standard_normal((M, E))
    nbr = O.top_K_neighbours(O.cosine_similarity(phi), K)
    assert np.array_equal(O.warmup_merge(phi, nbr, 0.0), phi)                       # alpha = 0
    d1 = O.warmup_merge(phi, nbr, 1.0) - phi
    np.testing.assert_allclose(O.warmup_merge(phi, nbr, 0.1) - phi, 0.1 * d1, rtol=1e-12, atol=1e-16)   # linear in alpha
    same = np.tile(phi[:1], (M, 1))
    np.testing.assert_allclose(O.warmup_merge(same, nbr, 0.7), same, rtol=1e-15)    # identical experts
    # K = M-1, alpha = 1: every expert becomes the mean of the others, all read before any is written
    nb_all = O.top_K_neighbours(O.cosine_similarity(phi), M - 1)
    want = (phi.sum(0, keepdims=True) - phi) / (M - 1)
    np.testing.assert_allclose(O.warmup_merge(phi, nb_all, 1.0), want, rtol=1e-12, atol=1e-15)
    # explicit loops
    out = O.warmup_merge(phi, nbr, 0.25)
    for j in range(M):
        for c in range(E):
            v = phi[j, c] + 0.25 / K * sum(phi[int(q), c] - phi[j, c] for q in nbr[j])
            assert abs(out[j, c] - v) < 1e-14

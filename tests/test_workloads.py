"""The seeded input generators: representability, determinism, margin rule, imbalance (CPU only)."""
import numpy as np

from oracle import spes_oracle as O
from spes_workloads import CONFIGS, MARGIN, bf16_bits, bf16_round, layer_inputs, merge_inputs, min_topk_gap


def test_bf16_round_is_rne_and_idempotent():
    a = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -7, -0.3, 3.0e38, 1e-40], dtype=np.float32)
    r = bf16_round(a)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0 + 2 ** -6 and r[3] == 1.0 + 2 ** -7   # ties to even
    assert np.array_equal(bf16_round(r), r)
    import torch
    big = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    assert np.array_equal(bf16_round(big), torch.from_numpy(big).bfloat16().float().numpy())
    assert np.array_equal(bf16_bits(bf16_round(big)), torch.from_numpy(big).bfloat16().view(torch.int16).numpy().view(np.uint16))


def test_layer_inputs_deterministic_and_margin():
    for name in ("cfg1", "cfg2_small", "cfg4_small"):
        cfg = CONFIGS[name]
        a = layer_inputs(cfg); b = layer_inputs(cfg)
        for key in ("x", "w_router", "w_gate", "w_down", "dy"):
            assert np.array_equal(a[key], b[key])
            if cfg.dtype == "bf16":
                assert np.array_equal(bf16_round(a[key]), a[key])
        assert a["trainable_mask"].sum() == cfg.n_trainable
        assert min_topk_gap(a["x"], a["w_router"], a["router_bias"], cfg.k).min() >= MARGIN
        s = O.router_logits(a["x"], a["w_router"], a["router_bias"])
        top = -np.sort(-s, axis=1)[:, :cfg.k + 1]
        assert np.min(top[:, :-1] - top[:, 1:]) >= MARGIN
    assert CONFIGS["cfg1"].renorm == 1 and layer_inputs(CONFIGS["cfg1"])["trainable_mask"].tolist() == [1, 1, 1, 1, 0, 0, 0, 0]


def test_upcycled_config_experts_are_near_copies():
    a = layer_inputs(CONFIGS["cfg4_small"])
    spread = np.abs(a["w_gate"] - a["w_gate"][0]).max()
    assert 0 < spread < 2e-3
    p = O.softmax(O.router_logits(a["x"], a["w_router"], None))
    assert p.max() < 2.5 / 32 and p.min() > 0.4 / 32          # near-uniform routing probabilities


def test_merge_inputs_structure():
    mi = merge_inputs(M=64, elems=16, n_nodes=16, experts_per_node=16, dtype="bf16", seed=20260216, need_zero_and_single=True)
    assert mi["trainer_count"].sum() == 256
    assert (mi["trainer_count"] == 0).any() and (mi["trainer_count"] == 1).any()
    for i, st in enumerate(mi["stores"]):
        assert st.shape == (16, 16) and np.array_equal(bf16_round(st), st)
        assert np.array_equal(np.nonzero(mi["slot"][i] >= 0)[0], mi["subsets"][i])

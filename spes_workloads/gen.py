"""Seeded synthetic workloads for the SPES MoE-layer hot path.

This module only *draws inputs*: tensors of the shapes, value distributions and
load-imbalance structure of an MoE feed-forward layer as trained by SPES
(Sec. 3.2 "Overall Framework", Sec. 3.3 "Expert Assignment and Local Training"),
plus node-local expert copies for the synchronisation step (Sec. 3.3 "Sparse
Synchronization").  It holds none of the layer's arithmetic.  The single piece
of linear algebra in here is the *acceptance test* on router margins (a matmul
followed by a sort), which decides whether a drawn token is kept; it produces no
value that either implementation consumes.

Every tensor is returned as float32 whose values are exactly representable in
the configuration's storage type (fp32, or bf16 after round-to-nearest-even), so
that an fp64 checker and a device kernel can both read the very same numbers.

All draws are counter-based (Philox keyed by (seed, tensor id, attempt)), so any
tensor can be regenerated independently of the others.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, Optional

import numpy as np

# ----------------------------------------------------------------------------
# storage-type helpers (no arithmetic of the method: value representation only)
# ----------------------------------------------------------------------------


def bf16_round(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    a = np.asarray(a, dtype=np.float32)
    return bf16_round(a) if dtype == "bf16" else a


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "value is not bf16-representable"
    return (u >> np.uint32(16)).astype(np.uint16)


# ----------------------------------------------------------------------------
# configurations
# ----------------------------------------------------------------------------


@dataclasses.dataclass(frozen=True)
class MoEConfig:
    name: str
    T: int            # tokens
    d: int            # d_model
    M: int            # experts
    f: int            # d_ff of one SwiGLU expert
    k: int            # top-k
    dtype: str        # "f32" | "bf16" (storage of params + activations)
    renorm: int       # 1: gates renormalised over the chosen k
    n_trainable: int
    trainable: str    # "first" | "random"
    bias: str         # "none" | "normal" | "gumbel"
    bias_scale: float
    router_sigma: float
    upcycled: bool    # experts = one dense FFN + tiny per-expert noise
    seed: int

    @property
    def R(self) -> int:
        return self.T * self.k


_BASE_SEED = 20260211

CONFIGS: Dict[str, MoEConfig] = {
    # the five measured workloads
    "cfg1": MoEConfig("cfg1", 512, 256, 8, 512, 2, "f32", 1, 4, "first", "none", 0.0, 0.02, False, _BASE_SEED + 1),
    "cfg2": MoEConfig("cfg2", 16384, 2048, 64, 1024, 8, "bf16", 0, 16, "random", "normal", 0.5, 0.02, False, _BASE_SEED + 2),
    "cfg3": MoEConfig("cfg3", 32768, 4096, 64, 1408, 8, "bf16", 0, 8, "random", "gumbel", 1.0, 0.02, False, _BASE_SEED + 3),
    "cfg4": MoEConfig("cfg4", 16384, 3584, 32, 4864, 2, "bf16", 1, 8, "random", "none", 0.0, 1e-3, True, _BASE_SEED + 4),
    "cfg5": MoEConfig("cfg5", 16384, 2048, 64, 1024, 8, "bf16", 0, 16, "random", "normal", 0.5, 0.02, False, _BASE_SEED + 5),
    # reduced shapes with the same structure, for element-by-element parity
    "cfg2_small": MoEConfig("cfg2_small", 1000, 256, 64, 192, 8, "bf16", 0, 16, "random", "normal", 0.5, 0.02, False, _BASE_SEED + 12),
    "cfg3_small": MoEConfig("cfg3_small", 1531, 512, 64, 352, 8, "bf16", 0, 8, "random", "gumbel", 1.0, 0.02, False, _BASE_SEED + 13),
    "cfg4_small": MoEConfig("cfg4_small", 777, 448, 32, 608, 2, "bf16", 1, 8, "random", "none", 0.0, 1e-3, True, _BASE_SEED + 14),
    "cfg1_bf16": MoEConfig("cfg1_bf16", 512, 256, 8, 512, 2, "bf16", 1, 4, "first", "none", 0.0, 0.02, False, _BASE_SEED + 15),
    # the layer shapes of the paper's own models (Sec. 4, model-configuration table) at one micro-batch of
    # 2 x 2048 tokens; trainable experts = experts / nodes of the corresponding experiment; the 9B model is upcycled
    "paper_1b": MoEConfig("paper_1b", 4096, 768, 16, 2048, 2, "bf16", 0, 4, "random", "none", 0.0, 0.02, False, _BASE_SEED + 21),
    "paper_2b": MoEConfig("paper_2b", 4096, 1536, 16, 1280, 2, "bf16", 0, 1, "random", "none", 0.0, 0.02, False, _BASE_SEED + 22),
    "paper_7b": MoEConfig("paper_7b", 4096, 2048, 32, 2048, 4, "bf16", 0, 8, "random", "none", 0.0, 0.02, False, _BASE_SEED + 23),
    "paper_9b": MoEConfig("paper_9b", 4096, 2048, 8, 6144, 2, "bf16", 1, 2, "random", "none", 0.0, 1e-3, True, _BASE_SEED + 24),
    "cfg2_f32": MoEConfig("cfg2_f32", 300, 128, 16, 96, 4, "f32", 0, 5, "random", "normal", 0.5, 0.02, False, _BASE_SEED + 16),
}

MARGIN = 1e-3          # minimum gap between adjacent sorted top-(k+1) router logits
_MAX_ATTEMPTS = 64

# tensor ids for the Philox key
_ID = dict(x=1, w_router=2, bias=3, w_gate=4, w_up=5, w_down=6, dy=7, mask=8,
           dense=9, subsets=10, node_noise=11, node_weight=12)


def _rng(seed: int, tensor: str, sub: int = 0, attempt: int = 0) -> np.random.Generator:
    key = [np.uint64(seed), np.uint64((_ID[tensor] << 40) | (sub << 8) | attempt)]
    return np.random.Generator(np.random.Philox(key=key))


def _normal(seed, tensor, shape, sigma, sub=0, attempt=0) -> np.ndarray:
    a = _rng(seed, tensor, sub, attempt).standard_normal(shape, dtype=np.float32)
    if sigma != 1.0:
        a *= np.float32(sigma)
    return a


def _parallel_experts(fn, M: int) -> list:
    with ThreadPoolExecutor(max_workers=8) as ex:
        return list(ex.map(fn, range(M)))


# ----------------------------------------------------------------------------
# acceptance test on router margins
# ----------------------------------------------------------------------------


def min_topk_gap(x: np.ndarray, w_router: np.ndarray, bias: Optional[np.ndarray], k: int) -> np.ndarray:
    """Per token: smallest gap between adjacent entries of the sorted top-(k+1) scores.

    Evaluated in fp64 on the stored (already rounded) values.  Used only to accept
    or reject a drawn token, so that the identity *and order* of its k selected
    experts do not hinge on rounding.
    """
    s = x.astype(np.float64) @ w_router.astype(np.float64).T
    if bias is not None:
        s = s + bias.astype(np.float64)[None, :]
    M = s.shape[1]
    top = -np.sort(-s, axis=1)[:, : min(k + 1, M)]
    if top.shape[1] < 2:
        return np.full(s.shape[0], np.inf)
    return np.min(top[:, :-1] - top[:, 1:], axis=1)


# ----------------------------------------------------------------------------
# layer inputs
# ----------------------------------------------------------------------------


def expert_weights(cfg: MoEConfig, which: str) -> np.ndarray:
    """One of w_gate [M,f,d], w_up [M,f,d], w_down [M,d,f] for a configuration."""
    shape = (cfg.d, cfg.f) if which == "w_down" else (cfg.f, cfg.d)
    if cfg.upcycled:
        sub0 = {"w_gate": 0, "w_up": 1, "w_down": 2}[which]
        dense = _normal(cfg.seed, "dense", shape, 0.02, sub=sub0)

        def one(e):
            noise = _normal(cfg.seed, which, shape, 1e-4, sub=e)
            return to_storage(dense + noise, cfg.dtype)
    else:
        def one(e):
            return to_storage(_normal(cfg.seed, which, shape, 0.02, sub=e), cfg.dtype)
    out = np.empty((cfg.M,) + shape, dtype=np.float32)

    def fill(e):
        out[e] = one(e)
    _parallel_experts(fill, cfg.M)
    return out


def router_bias(cfg: MoEConfig) -> Optional[np.ndarray]:
    """Per-expert logit bias (fp32) that induces load imbalance; None if the config has none."""
    if cfg.bias == "none":
        return None
    g = _rng(cfg.seed, "bias")
    if cfg.bias == "normal":
        return (g.standard_normal(cfg.M) * cfg.bias_scale).astype(np.float32)
    if cfg.bias == "gumbel":
        u = g.random(cfg.M)
        return (-np.log(-np.log(u)) * cfg.bias_scale).astype(np.float32)
    raise ValueError(cfg.bias)


def trainable_mask(cfg: MoEConfig) -> np.ndarray:
    m = np.zeros(cfg.M, dtype=np.uint8)
    if cfg.trainable == "first":
        m[: cfg.n_trainable] = 1
    else:
        sel = _rng(cfg.seed, "mask").permutation(cfg.M)[: cfg.n_trainable]
        m[sel] = 1
    return m


def tokens_with_margin(cfg: MoEConfig, w_router: np.ndarray, bias: Optional[np.ndarray], micro: int = 0):
    """x [T,d] ~ N(0,1) in storage precision; tokens whose router margin is < MARGIN are redrawn.
    `micro` selects an independent stream (micro-batch number) under the same seed."""
    x = to_storage(_normal(cfg.seed, "x", (cfg.T, cfg.d), 1.0, sub=micro), cfg.dtype)
    redraws = 0
    bad = np.nonzero(min_topk_gap(x, w_router, bias, cfg.k) < MARGIN)[0]
    attempt = 1
    while bad.size:
        if attempt >= _MAX_ATTEMPTS:
            raise RuntimeError(f"{cfg.name}: {bad.size} tokens still below margin after {attempt} attempts")
        redraws += bad.size
        # one fresh stream per attempt; row i of the attempt replaces token bad[i]
        fresh = to_storage(_normal(cfg.seed, "x", (bad.size, cfg.d), 1.0, sub=micro, attempt=attempt), cfg.dtype)
        x[bad] = fresh
        still = min_topk_gap(fresh, w_router, bias, cfg.k) < MARGIN
        bad = bad[still]
        attempt += 1
    return x, redraws


def layer_inputs(cfg: MoEConfig, weights: bool = True, micro: int = 0) -> dict:
    """All inputs of one fwd+bwd pass of the layer for `cfg`.

    Keys: x [T,d], w_router [M,d], router_bias [M] or None, w_gate/w_up [M,f,d],
    w_down [M,d,f], dy [T,d], trainable_mask uint8 [M], redraw_fraction.
    `micro` > 0 gives another micro-batch (x, dy) for the same weights.
    """
    w_router = to_storage(_normal(cfg.seed, "w_router", (cfg.M, cfg.d), cfg.router_sigma), cfg.dtype)
    bias = router_bias(cfg)
    x, redraws = tokens_with_margin(cfg, w_router, bias, micro)
    out = dict(cfg=cfg, x=x, w_router=w_router, router_bias=bias,
               dy=to_storage(_normal(cfg.seed, "dy", (cfg.T, cfg.d), 1.0, sub=micro), cfg.dtype),
               trainable_mask=trainable_mask(cfg), redraw_fraction=redraws / cfg.T)
    if weights:
        for w in ("w_gate", "w_up", "w_down"):
            out[w] = expert_weights(cfg, w)
    return out


def custom_config(name="custom", **kw) -> MoEConfig:
    base = dict(T=64, d=32, M=4, f=48, k=2, dtype="f32", renorm=0, n_trainable=2, trainable="first",
                bias="none", bias_scale=0.0, router_sigma=0.02, upcycled=False, seed=_BASE_SEED + 100)
    base.update(kw)
    return MoEConfig(name, **base)


# ----------------------------------------------------------------------------
# synchronisation inputs: node-local copies of experts
# ----------------------------------------------------------------------------


def merge_inputs(M: int, elems: int, n_nodes: int, experts_per_node: Optional[int], dtype: str, seed: int,
                 noise: float = 1e-3, weighted: bool = True, base: Optional[np.ndarray] = None,
                 need_zero_and_single: bool = False) -> dict:
    """Node-local stores of trained experts for one parameter matrix.

    base [M,elems] is the previous global value.  Node i trained the experts in
    subset_i (ascending ids; all M if experts_per_node is None) and holds
    base[subset_i] + N(0,noise) in storage precision.  slot[i,j] is the row of
    expert j in node i's store, or -1.  node_weight ~ U[0.5,1.5] (or None = uniform).
    With need_zero_and_single the subsets are redrawn (attempt counter in the key)
    until some expert has no trainer and some expert exactly one.
    """
    if base is None:
        base = to_storage(_normal(seed, "dense", (M, elems), 0.02, sub=7), dtype)
    attempt = 0
    while True:
        slot = np.full((n_nodes, M), -1, dtype=np.int32)
        subsets = []
        for i in range(n_nodes):
            if experts_per_node is None:
                sub = np.arange(M)
            else:
                sub = np.sort(_rng(seed, "subsets", sub=i, attempt=attempt).permutation(M)[:experts_per_node])
            subsets.append(sub)
            slot[i, sub] = np.arange(sub.size, dtype=np.int32)
        cnt = (slot >= 0).sum(axis=0)
        if not need_zero_and_single or (np.any(cnt == 0) and np.any(cnt == 1)):
            break
        attempt += 1
        if attempt >= _MAX_ATTEMPTS:
            raise RuntimeError("no subset draw with an untrained and a singly-trained expert")
    stores = []
    for i, sub in enumerate(subsets):
        n = _normal(seed, "node_noise", (sub.size, elems), noise, sub=i)
        stores.append(to_storage(base[sub] + n, dtype))
    w = None
    if weighted:
        w = (0.5 + _rng(seed, "node_weight").random(n_nodes)).astype(np.float32)
    return dict(base=base, stores=stores, slot=slot, node_weight=w, subsets=subsets, trainer_count=cnt.astype(np.int32))

"""Device buffers of one routed feed-forward layer and the calls that run it: a convenience holder for tests, the smoke
check and the benchmark.  Marshalling only -- every step of the path runs in the library's kernels."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as S


def to_dev(a: np.ndarray, dtype: str, device) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)          # exact: the generator already rounded to bf16
    return t.to(device)


def shape_of(cfg) -> "S.spes_moe_shape":
    return S.moe_shape(cfg.T, cfg.d, cfg.M, cfg.f, cfg.k, S.SPES_F32 if cfg.dtype == "f32" else S.SPES_BF16, cfg.renorm)


class DeviceLayer:
    """Device copies of one layer's inputs plus the output/ctx buffers of fwd and bwd."""

    def __init__(self, inp: dict, device, mask=None):
        cfg = inp["cfg"]
        self.cfg, self.shape, self.dev = cfg, shape_of(cfg), device
        dt = cfg.dtype
        self.x = to_dev(inp["x"], dt, device); self.dy = to_dev(inp["dy"], dt, device)
        self.w_router = to_dev(inp["w_router"], dt, device)
        self.bias = None if inp["router_bias"] is None else torch.from_numpy(inp["router_bias"]).to(device)
        self.w_gate = to_dev(inp["w_gate"], dt, device); self.w_up = to_dev(inp["w_up"], dt, device)
        self.w_down = to_dev(inp["w_down"], dt, device)
        st = S.torch_dtype(self.shape.dtype)
        T, d, M, f, k = cfg.T, cfg.d, cfg.M, cfg.f, cfg.k
        self.y = torch.empty(T, d, dtype=st, device=device)
        self.idx = torch.empty(T, k, dtype=torch.int32, device=device)
        self.gate = torch.empty(T, k, dtype=torch.float32, device=device)
        self.count = torch.empty(M, dtype=torch.int32, device=device)
        self.ctx = torch.empty(S.spes_moe_ctx_bytes(self.shape), dtype=torch.uint8, device=device)
        self.dx = torch.empty(T, d, dtype=st, device=device)
        self.d_w_router = torch.zeros(M, d, dtype=torch.float32, device=device)
        self.set_mask(inp["trainable_mask"] if mask is None else mask)

    def set_mask(self, mask):
        cfg = self.cfg
        self.mask = np.asarray(mask, dtype=np.uint8)
        n = int(self.mask.sum())
        self.trainable = [int(e) for e in np.nonzero(self.mask)[0]]
        mk = lambda *s: torch.zeros(*s, dtype=torch.float32, device=self.dev) if n else None
        self.d_w_gate, self.d_w_up, self.d_w_down = mk(n, cfg.f, cfg.d), mk(n, cfg.f, cfg.d), mk(n, cfg.d, cfg.f)

    def fwd(self):
        S.spes_moe_fwd(self.shape, self.x, self.w_router, self.bias, self.w_gate, self.w_up, self.w_down, self.y, self.idx,
                       self.gate, self.count, self.ctx)

    def bwd(self, accumulate=0):
        S.spes_moe_bwd(self.shape, self.dy, self.x, self.w_router, self.w_gate, self.w_up, self.w_down, self.ctx, self.mask,
                       self.dx, self.d_w_router, self.d_w_gate, self.d_w_up, self.d_w_down, accumulate)

    def aux(self, lb_coef, z_coef, grad_scale=1.0):
        """Router auxiliary losses of the last forward; arms the next bwd.  Returns (L_lb, L_z)."""
        losses = torch.zeros(2, dtype=torch.float32, device=self.dev)
        S.spes_moe_router_aux(self.shape, self.ctx, lb_coef, z_coef, grad_scale, losses)
        return tuple(float(v) for v in losses.cpu().numpy())

    def permuted(self):
        """The dispatched copy of x in expert-contiguous order, from the routing tables of the last forward."""
        xp = torch.empty(self.cfg.T * self.cfg.k, self.cfg.d, dtype=self.x.dtype, device=self.dev)
        S.spes_moe_permute(self.shape, self.x, self.ctx, xp)
        return xp

    def grad_scatter(self):
        """The stand-alone backward of the combine: (dyp [T*k, d], dgate [T, k]) from dy and the last forward's record."""
        dyp = torch.empty(self.cfg.T * self.cfg.k, self.cfg.d, dtype=self.x.dtype, device=self.dev)
        dgate = torch.empty(self.cfg.T, self.cfg.k, dtype=torch.float32, device=self.dev)
        S.spes_moe_grad_scatter(self.shape, self.dy, self.ctx, dyp, dgate)
        return dyp, dgate

    def view(self, name):
        return S.ctx_view(self.shape, self.ctx, name)

    def host(self, t):
        return t.float().cpu().numpy() if t.dtype == torch.bfloat16 else t.cpu().numpy()

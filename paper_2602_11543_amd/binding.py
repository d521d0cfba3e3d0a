"""ctypes binding of libspes.so: argument marshalling only.

Every function has the name and argument order of its C entry point in
include/spes.h (include/spes_bench.h for the benchmark aids) and takes torch tensors (device memory) or numpy arrays (host
arrays) in place of raw pointers.  Nothing is computed here; if the library is
missing and cannot be built the import fails loudly -- there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np
import torch

from . import build as _build

SPES_F32, SPES_BF16 = 0, 1


class SpesError(RuntimeError):
    pass


class spes_moe_shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("T", "d_model", "n_experts", "d_ff", "top_k", "dtype", "renorm_topk")]


_LAYOUT_FIELDS = ("total", "logits", "lse", "topk_idx", "topk_gate", "offset", "perm", "inv", "a", "b", "h", "yp",
                  "dlogits", "dgate")


class spes_moe_ctx_layout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_size_t) for n in _LAYOUT_FIELDS]


def _load() -> ctypes.CDLL:
    if not os.path.exists(_build.LIB):
        _build.build_library(verbose=False)      # raises if hipcc is unavailable
    lib = ctypes.CDLL(_build.LIB)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    shp = ctypes.POINTER(spes_moe_shape)
    lib.spes_moe_ctx_bytes.restype = sz
    lib.spes_moe_ctx_bytes.argtypes = [shp]
    lib.spes_moe_ctx_describe.restype = i32
    lib.spes_moe_ctx_describe.argtypes = [shp, ctypes.POINTER(spes_moe_ctx_layout)]
    lib.spes_moe_fwd.restype = i32
    lib.spes_moe_fwd.argtypes = [shp] + [vp] * 12
    lib.spes_moe_bwd.restype = i32
    lib.spes_moe_bwd.argtypes = [shp] + [vp] * 13 + [i32, vp]
    lib.spes_moe_permute.restype = i32
    lib.spes_moe_permute.argtypes = [shp, vp, vp, vp, vp]
    lib.spes_moe_grad_scatter.restype = i32
    lib.spes_moe_grad_scatter.argtypes = [shp, vp, vp, vp, vp, vp]
    lib.spes_moe_router_aux.restype = i32
    lib.spes_moe_router_aux.argtypes = [shp, vp, ctypes.c_float, ctypes.c_float, ctypes.c_float, vp, vp]
    lib.spes_masked_adamw.restype = i32
    lib.spes_masked_adamw.argtypes = [i32, i64, i32, vp, vp, vp, vp, vp, vp] + [ctypes.c_float] * 5 + [i32, ctypes.c_float, vp]
    lib.spes_upcycle_init.restype = i32
    lib.spes_upcycle_init.argtypes = [i32, i64, i32, vp, ctypes.c_float, ctypes.c_float, ctypes.c_uint64, ctypes.c_uint64, vp, vp]
    lib.spes_expert_pack.restype = i32
    lib.spes_expert_pack.argtypes = [i32, i64, i32, vp, vp, vp, i32, vp]
    lib.spes_expert_merge.restype = i32
    lib.spes_expert_merge.argtypes = [i32, i64, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.spes_warmup_scratch_bytes.restype = sz
    lib.spes_warmup_scratch_bytes.argtypes = [i32, i64]
    lib.spes_expert_warmup_merge.restype = i32
    lib.spes_expert_warmup_merge.argtypes = [i32, i32, i32, ctypes.c_float, vp, i64, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.spes_expert_warmup_merge_static.restype = i32
    lib.spes_expert_warmup_merge_static.argtypes = [i32, i32, i32, ctypes.c_float, vp, i64, i32, vp, vp, vp, vp, vp, vp]
    lib.spes_ref_mfma_rate.restype = i32
    lib.spes_ref_mfma_rate.argtypes = [vp, i32, i32, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.spes_profile_enable.restype = i32
    lib.spes_profile_enable.argtypes = [i32]
    lib.spes_profile_read.restype = i32
    lib.spes_profile_read.argtypes = [i32, vp, vp, i32]
    lib.spes_strerror.restype = ctypes.c_char_p
    lib.spes_strerror.argtypes = [i32]
    return lib


_lib = _load()


def library_path() -> str:
    return _build.LIB


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise SpesError(f"{what}: {_lib.spes_strerror(rc).decode()} (code {rc})")


def _dev(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise SpesError("device arguments must be contiguous GPU tensors")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    return ctypes.c_void_p(int(stream))


def torch_dtype(dtype: int) -> torch.dtype:
    return torch.float32 if dtype == SPES_F32 else torch.bfloat16


def moe_shape(T, d_model, n_experts, d_ff, top_k, dtype, renorm_topk) -> spes_moe_shape:
    return spes_moe_shape(T, d_model, n_experts, d_ff, top_k, dtype, renorm_topk)


def spes_strerror(code: int) -> str:
    return _lib.spes_strerror(code).decode()


def spes_moe_ctx_bytes(shape: spes_moe_shape) -> int:
    return int(_lib.spes_moe_ctx_bytes(ctypes.byref(shape)))


def spes_moe_ctx_describe(shape: spes_moe_shape) -> dict:
    lay = spes_moe_ctx_layout()
    _check(_lib.spes_moe_ctx_describe(ctypes.byref(shape), ctypes.byref(lay)), "spes_moe_ctx_describe")
    return {n: int(getattr(lay, n)) for n in _LAYOUT_FIELDS}


def spes_moe_fwd(shape, x, w_router, router_bias, w_gate, w_up, w_down, y, topk_idx, topk_gate, expert_count, ctx,
                 stream=None) -> None:
    _check(_lib.spes_moe_fwd(ctypes.byref(shape), _dev(x), _dev(w_router), _dev(router_bias), _dev(w_gate), _dev(w_up),
                             _dev(w_down), _dev(y), _dev(topk_idx), _dev(topk_gate), _dev(expert_count), _dev(ctx),
                             _stream(stream)), "spes_moe_fwd")


def spes_moe_bwd(shape, dy, x, w_router, w_gate, w_up, w_down, ctx, trainable_mask, dx, d_w_router, d_w_gate, d_w_up,
                 d_w_down, accumulate=0, stream=None) -> None:
    mask = np.ascontiguousarray(trainable_mask, dtype=np.uint8)
    if mask.shape != (shape.n_experts,):
        raise SpesError("trainable_mask must have one byte per expert")
    _check(_lib.spes_moe_bwd(ctypes.byref(shape), _dev(dy), _dev(x), _dev(w_router), _dev(w_gate), _dev(w_up), _dev(w_down),
                             _dev(ctx), mask.ctypes.data_as(ctypes.c_void_p), _dev(dx), _dev(d_w_router), _dev(d_w_gate),
                             _dev(d_w_up), _dev(d_w_down), int(accumulate), _stream(stream)), "spes_moe_bwd")


def spes_moe_permute(shape, x, ctx, xp, stream=None) -> None:
    _check(_lib.spes_moe_permute(ctypes.byref(shape), _dev(x), _dev(ctx), _dev(xp), _stream(stream)), "spes_moe_permute")


def spes_moe_grad_scatter(shape, dy, ctx, dyp, dgate, stream=None) -> None:
    _check(_lib.spes_moe_grad_scatter(ctypes.byref(shape), _dev(dy), _dev(ctx), _dev(dyp), _dev(dgate), _stream(stream)),
           "spes_moe_grad_scatter")


def spes_moe_router_aux(shape, ctx, lb_coef, z_coef, grad_scale, losses, stream=None) -> None:
    _check(_lib.spes_moe_router_aux(ctypes.byref(shape), _dev(ctx), float(lb_coef), float(z_coef), float(grad_scale),
                                    _dev(losses), _stream(stream)), "spes_moe_router_aux")


def spes_masked_adamw(n_experts, elems, dtype, param, trainable_mask, master, m, v, grad, lr, beta1, beta2, eps, weight_decay,
                      step, grad_scale=1.0, stream=None) -> None:
    mask = np.ascontiguousarray(trainable_mask, dtype=np.uint8)
    if mask.shape != (n_experts,):
        raise SpesError("trainable_mask must have one byte per expert")
    _check(_lib.spes_masked_adamw(n_experts, elems, dtype, _dev(param), mask.ctypes.data_as(ctypes.c_void_p), _dev(master),
                                  _dev(m), _dev(v), _dev(grad), float(lr), float(beta1), float(beta2), float(eps),
                                  float(weight_decay), int(step), float(grad_scale), _stream(stream)), "spes_masked_adamw")


def spes_upcycle_init(n_experts, elems, dtype, dense, fraction, sigma, seed, stream_id, out, stream=None) -> None:
    _check(_lib.spes_upcycle_init(n_experts, elems, dtype, _dev(dense), float(fraction), float(sigma), int(seed), int(stream_id),
                                  _dev(out), _stream(stream)), "spes_upcycle_init")


def spes_expert_pack(n_experts, elems, dtype, store, trainable_mask, packed, to_store=0, stream=None) -> None:
    mask = np.ascontiguousarray(trainable_mask, dtype=np.uint8)
    if mask.shape != (n_experts,):
        raise SpesError("trainable_mask must have one byte per expert")
    _check(_lib.spes_expert_pack(n_experts, elems, dtype, _dev(store), mask.ctypes.data_as(ctypes.c_void_p), _dev(packed),
                                 int(to_store), _stream(stream)), "spes_expert_pack")


def spes_expert_merge(n_experts, elems, dtype, node_store: Sequence[Optional[torch.Tensor]], slot, node_weight, dst,
                      trainer_count=None, stream=None) -> None:
    n_nodes = len(node_store)
    slot = np.ascontiguousarray(slot, dtype=np.int32)
    if slot.shape != (n_nodes, n_experts):
        raise SpesError("slot must be [n_nodes, n_experts]")
    ptrs = (ctypes.c_void_p * max(n_nodes, 1))(*[None if t is None else _dev(t).value for t in node_store])
    w = None if node_weight is None else np.ascontiguousarray(node_weight, dtype=np.float32)
    _check(_lib.spes_expert_merge(n_experts, elems, dtype, n_nodes, ctypes.cast(ptrs, ctypes.c_void_p),
                                  slot.ctypes.data_as(ctypes.c_void_p),
                                  None if w is None else w.ctypes.data_as(ctypes.c_void_p), _dev(dst),
                                  _dev(trainer_count), _stream(stream)), "spes_expert_merge")


def spes_warmup_scratch_bytes(n_experts: int, elems_in: int) -> int:
    return int(_lib.spes_warmup_scratch_bytes(n_experts, elems_in))


def spes_expert_warmup_merge(n_experts, dtype, top_K, alpha, w_in, elems_in, src: Sequence[torch.Tensor],
                             dst: Sequence[torch.Tensor], elems: Sequence[int], sim, nbr, scratch, stream=None) -> None:
    n_mats = len(src)
    sp = (ctypes.c_void_p * max(n_mats, 1))(*[_dev(t).value for t in src])
    dp = (ctypes.c_void_p * max(n_mats, 1))(*[_dev(t).value for t in dst])
    el = np.ascontiguousarray(elems, dtype=np.int64)
    _check(_lib.spes_expert_warmup_merge(n_experts, dtype, top_K, ctypes.c_float(alpha), _dev(w_in), elems_in, n_mats,
                                         ctypes.cast(sp, ctypes.c_void_p), ctypes.cast(dp, ctypes.c_void_p),
                                         el.ctypes.data_as(ctypes.c_void_p), _dev(sim), _dev(nbr), _dev(scratch),
                                         _stream(stream)), "spes_expert_warmup_merge")


def spes_expert_warmup_merge_static(n_experts, dtype, top_K, alpha, w_in, elems_in, src: Sequence[torch.Tensor],
                                    dst: Sequence[torch.Tensor], elems: Sequence[int], sim, nbr, stream=None) -> None:
    n_mats = len(src)
    sp = (ctypes.c_void_p * max(n_mats, 1))(*[_dev(t).value for t in src])
    dp = (ctypes.c_void_p * max(n_mats, 1))(*[_dev(t).value for t in dst])
    el = np.ascontiguousarray(elems, dtype=np.int64)
    _check(_lib.spes_expert_warmup_merge_static(n_experts, dtype, top_K, ctypes.c_float(alpha), _dev(w_in), elems_in, n_mats,
                                                ctypes.cast(sp, ctypes.c_void_p), ctypes.cast(dp, ctypes.c_void_p),
                                                el.ctypes.data_as(ctypes.c_void_p), _dev(sim), _dev(nbr), _stream(stream)),
           "spes_expert_warmup_merge_static")


def spes_profile_enable(on: bool) -> None:
    _check(_lib.spes_profile_enable(1 if on else 0), "spes_profile_enable")


def spes_profile_read(which: int) -> list:
    """[(stage name, milliseconds)] of the latest forward (0) or backward (1) while stage timing is enabled."""
    cap = 24
    ms = (ctypes.c_float * cap)()
    names = (ctypes.c_char_p * cap)()
    n = _lib.spes_profile_read(which, ctypes.cast(ms, ctypes.c_void_p), ctypes.cast(names, ctypes.c_void_p), cap)
    if n < 0:
        _check(n, "spes_profile_read")
    return [(names[i].decode(), float(ms[i])) for i in range(n)]


def spes_ref_mfma_rate(data, blocks, iters, sink, stream=None) -> float:
    """Launches the register-resident MFMA loop; returns the floating-point operations it performs."""
    flop = ctypes.c_double(0.0)
    _check(_lib.spes_ref_mfma_rate(_dev(data), int(blocks), int(iters), _dev(sink), ctypes.byref(flop), _stream(stream)),
           "spes_ref_mfma_rate")
    return float(flop.value)


def ctx_view(shape: spes_moe_shape, ctx: torch.Tensor, name: str) -> torch.Tensor:
    """A typed view of one region of the context buffer (for inspection by tests)."""
    lay = spes_moe_ctx_describe(shape)
    T, d, M, f, k = shape.T, shape.d_model, shape.n_experts, shape.d_ff, shape.top_k
    R = T * k
    st = torch_dtype(shape.dtype)
    spec = dict(logits=(torch.float32, (T, M)), lse=(torch.float32, (T,)), topk_idx=(torch.int32, (T, k)),
                topk_gate=(torch.float32, (T, k)), offset=(torch.int32, (M + 1,)), perm=(torch.int32, (R,)),
                inv=(torch.int32, (R,)), a=(st, (R, f)), b=(st, (R, f)), h=(st, (R, f)), yp=(st, (R, d)),
                dlogits=(torch.float32, (T, M)), dgate=(torch.float32, (T, k)))[name]
    n = int(np.prod(spec[1])) * torch.empty((), dtype=spec[0]).element_size()
    return ctx[lay[name]: lay[name] + n].view(spec[0]).view(spec[1])

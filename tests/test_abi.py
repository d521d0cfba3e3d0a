"""The C-ABI library loads and exports every entry point the header declares (no GPU needed)."""
import ctypes
import os
import re

import paper_2602_11543_amd as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_symbols_are_exported():
    inc = os.path.join(ROOT, "include")
    header = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    names = set(re.findall(r"SPES_API[^;(]*?\b(spes_\w+)\s*\(", header))
    assert {"spes_moe_grad_scatter", "spes_profile_enable", "spes_ref_mfma_rate"} <= names
    assert {"spes_moe_fwd", "spes_moe_bwd", "spes_expert_merge", "spes_expert_warmup_merge"} <= names
    lib = ctypes.CDLL(S.library_path())
    for n in names:
        assert hasattr(lib, n), n


def test_host_only_queries():
    sh = S.moe_shape(512, 256, 8, 512, 2, S.SPES_F32, 1)
    lay = S.spes_moe_ctx_describe(sh)
    assert lay["total"] == S.spes_moe_ctx_bytes(sh) > 0
    offs = sorted(v for k, v in lay.items() if k != "total")
    assert all(o % 256 == 0 for o in offs) and len(set(offs)) == len(offs)
    assert S.spes_moe_ctx_bytes(S.moe_shape(512, 256, 65, 512, 2, 0, 0)) == 0       # more than 64 experts
    assert S.spes_moe_ctx_bytes(S.moe_shape(512, 250, 8, 512, 2, 0, 0)) == 0        # d_model not a multiple of 8
    assert S.spes_warmup_scratch_bytes(8, 4096) > 0
    assert "aligned" in S.spes_strerror(-3)


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2602_11543_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text, f


def _fake(addr):
    return ctypes.c_void_p(addr)


def test_argument_checks_run_before_any_launch():
    """Bad arguments are rejected on the host: these calls never reach the GPU (none is needed to run them)."""
    lib = ctypes.CDLL(S.library_path())
    lib.spes_moe_fwd.restype = ctypes.c_int32
    lib.spes_moe_bwd.restype = ctypes.c_int32
    lib.spes_expert_merge.restype = ctypes.c_int32
    lib.spes_expert_warmup_merge.restype = ctypes.c_int32
    ok_shape = S.moe_shape(64, 64, 8, 64, 2, S.SPES_BF16, 0)
    p = [_fake(0x10000 + 0x1000 * i) for i in range(12)]           # aligned, never dereferenced
    fwd = lambda shape, ptrs: lib.spes_moe_fwd(ctypes.byref(shape), *ptrs, None)
    assert fwd(S.moe_shape(64, 64, 8, 64, 9, 1, 0), p[:11]) == -1          # top_k > n_experts
    assert fwd(S.moe_shape(64, 64, 8, 64, 2, 7, 0), p[:11]) == -1          # unknown dtype
    assert fwd(S.moe_shape(64, 64, 128, 64, 2, 1, 0), p[:11]) == -2        # more than 64 experts
    assert fwd(S.moe_shape(64, 60, 8, 64, 2, 1, 0), p[:11]) == -2          # d_model not a multiple of 8
    assert fwd(S.moe_shape(1 << 20, 4096, 8, 64, 2, 1, 0), p[:11]) == -2   # x beyond the 32-bit operand offsets of the bf16 path
    assert fwd(S.moe_shape(64, 8192, 64, 8192, 2, 1, 0), p[:11]) == -2     # expert weight tensor likewise
    nulls = list(p[:11]); nulls[5] = None
    assert fwd(ok_shape, nulls) == -1                                       # null y
    nulls = list(p[:11]); nulls[2] = None
    odd = list(p[:11]); odd[0] = _fake(0x10008)
    assert fwd(ok_shape, odd) == -3                                         # misaligned x (null bias is allowed)
    mask = (ctypes.c_uint8 * 8)(1, 0, 0, 0, 0, 0, 0, 0)
    bwd_args = [p[0], p[1], p[2], p[3], p[4], p[5], p[6], ctypes.cast(mask, ctypes.c_void_p), p[7], p[8], None, p[9], p[10]]
    assert lib.spes_moe_bwd(ctypes.byref(ok_shape), *bwd_args, 0, None) == -1   # a trainable expert but no d_w_gate buffer
    lib.spes_moe_permute.restype = ctypes.c_int32
    lib.spes_moe_permute.argtypes = [ctypes.c_void_p] * 5
    assert lib.spes_moe_permute(ctypes.byref(ok_shape), p[0], p[1], None, None) == -1                   # no output
    assert lib.spes_moe_permute(ctypes.byref(ok_shape), p[0], p[1], _fake(0x20004), None) == -3         # misaligned output
    assert lib.spes_moe_permute(ctypes.byref(S.moe_shape(64, 60, 8, 64, 2, 1, 0)), p[0], p[1], p[2], None) == -2
    lib.spes_ref_mfma_rate.restype = ctypes.c_int32
    lib.spes_ref_mfma_rate.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    assert lib.spes_ref_mfma_rate(p[0], 0, 10, p[1], None, None) == -1                                   # no blocks
    assert lib.spes_ref_mfma_rate(None, 4, 10, p[1], None, None) == -1                                   # no operands
    assert lib.spes_ref_mfma_rate(_fake(0x30008), 4, 10, p[1], None, None) == -3                         # misaligned operands
    lib.spes_moe_router_aux.restype = ctypes.c_int32
    lib.spes_moe_router_aux.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float, ctypes.c_float, ctypes.c_float,
                                        ctypes.c_void_p, ctypes.c_void_p]
    assert lib.spes_moe_router_aux(ctypes.byref(ok_shape), None, 0.01, 0.001, 1.0, p[0], None) == -1      # no ctx
    assert lib.spes_moe_router_aux(ctypes.byref(ok_shape), p[0], 0.01, 0.001, 1.0, None, None) == -1      # no output
    lib.spes_masked_adamw.restype = ctypes.c_int32
    lib.spes_masked_adamw.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int32] + [ctypes.c_void_p] * 6 + \
        [ctypes.c_float] * 5 + [ctypes.c_int32, ctypes.c_float, ctypes.c_void_p]
    m2 = ctypes.cast((ctypes.c_uint8 * 2)(1, 0), ctypes.c_void_p)
    adam = lambda elems, dtype, master, step, b1=0.9: lib.spes_masked_adamw(
        2, elems, dtype, p[0], m2, master, p[2], p[3], p[4], 5e-4, b1, 0.95, 1e-8, 0.1, step, 1.0, None)
    assert adam(64, 1, None, 1) == -1             # a bf16 store needs fp32 weights
    assert adam(64, 1, p[1], 0) == -1             # steps count from 1
    assert adam(64, 1, p[1], 1, b1=1.0) == -1     # beta must be below 1
    assert adam(60, 1, p[1], 1) == -2             # elems not a multiple of 8
    lib.spes_upcycle_init.restype = ctypes.c_int32
    lib.spes_upcycle_init.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_float,
                                      ctypes.c_float, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p]
    assert lib.spes_upcycle_init(4, 64, 1, p[0], 1.5, 0.02, 1, 0, p[1], None) == -1      # fraction above 1
    assert lib.spes_upcycle_init(4, 60, 1, p[0], 0.5, 0.02, 1, 0, p[1], None) == -2      # elems not a multiple of 8
    assert lib.spes_upcycle_init(4, 64, 1, _fake(0x10008), 0.5, 0.02, 1, 0, p[1], None) == -3
    lib.spes_expert_pack.restype = ctypes.c_int32
    lib.spes_expert_pack.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                     ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p]
    assert lib.spes_expert_pack(2, 64, 1, p[0], m2, None, 0, None) == -1                 # a trainable expert but no buffer
    assert lib.spes_expert_pack(2, 60, 1, p[0], m2, p[1], 0, None) == -2
    slot = (ctypes.c_int32 * 4)(0, -1, -1, 0)
    stores = (ctypes.c_void_p * 2)(0x20000, 0x30000)
    args = lambda elems, dtype: (2, ctypes.c_int64(elems), dtype, 2, ctypes.cast(stores, ctypes.c_void_p),
                                 ctypes.cast(slot, ctypes.c_void_p), None, p[0], None, None)
    assert lib.spes_expert_merge(*args(100, 1)) == -2                       # elems not a multiple of 8
    assert lib.spes_expert_merge(*args(128, 5)) == -1                       # unknown dtype
    assert lib.spes_expert_warmup_merge(8, 1, 8, ctypes.c_float(0.1), p[0], ctypes.c_int64(64), 0, None, None, None, None,
                                        p[1], p[2], None) == -1            # top_K must be < n_experts

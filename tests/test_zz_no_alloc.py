"""The warm-up merge entry point that allocates nothing (its Gram partials live in the library's own device image)
against the entry point with a caller-provided scratch, through the C ABI: two calls in a row, the second smaller."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2602_11543_amd as S
from spes_workloads import bf16_round

pytestmark = pytest.mark.gpu


def _experts(M, E, dtype, seed):
    rng = np.random.default_rng(seed)
    centres = rng.standard_normal((4, E))
    w = np.stack([centres[j % 4] + (0.15 + 0.05 * j) * rng.standard_normal(E) for j in range(M)]).astype(np.float32) * 0.02
    return bf16_round(w) if dtype == "bf16" else w


def _dev(a, dtype, device):
    t = torch.from_numpy(np.ascontiguousarray(a))
    return (t.to(torch.bfloat16) if dtype == "bf16" else t).to(device)


def _ptrs(ts):
    return ctypes.cast((ctypes.c_void_p * len(ts))(*[t.data_ptr() for t in ts]), ctypes.c_void_p)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_scratch_entry_matches_the_caller_scratch_entry(dtype, device):
    lib = ctypes.CDLL(S.library_path())
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.spes_expert_warmup_merge.restype = i32
    lib.spes_expert_warmup_merge.argtypes = [i32, i32, i32, ctypes.c_float, vp, i64, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.spes_expert_warmup_merge_static.restype = i32
    lib.spes_expert_warmup_merge_static.argtypes = [i32, i32, i32, ctypes.c_float, vp, i64, i32, vp, vp, vp, vp, vp, vp]
    lib.spes_warmup_scratch_bytes.restype = ctypes.c_size_t
    lib.spes_warmup_scratch_bytes.argtypes = [i32, i64]
    dt = S.SPES_F32 if dtype == "f32" else S.SPES_BF16
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    # the first problem fills many chunks of the static buffer, the second (smaller in every way) only a few of them
    for M, E, K, alpha in ((48, 40 * 4096 + 64, 4, 0.1), (12, 2 * 4096 + 8, 3, 0.5)):
        print(f"[case] static-scratch warm-up merge {dtype} M={M} E={E}", flush=True)
        mats = [_experts(M, E, dtype, 31 + M), _experts(M, 776, dtype, 32 + M)]
        src = [_dev(m, dtype, device) for m in mats]
        elems = (ctypes.c_int64 * 2)(E, 776)
        outs = []
        for static in (False, True):
            dst = [torch.full_like(t, 7.0) for t in src]
            sim = torch.full((M, M), float("nan"), dtype=torch.float32, device=device)
            nbr = torch.full((M, K), -1, dtype=torch.int32, device=device)
            common = (M, dt, K, ctypes.c_float(alpha), src[0].data_ptr(), E, 2, _ptrs(src), _ptrs(dst),
                      ctypes.cast(elems, ctypes.c_void_p), sim.data_ptr(), nbr.data_ptr())
            if static:
                rc = lib.spes_expert_warmup_merge_static(*common, stream)
            else:
                scratch = torch.empty(lib.spes_warmup_scratch_bytes(M, E), dtype=torch.uint8, device=device)
                rc = lib.spes_expert_warmup_merge(*common, scratch.data_ptr(), stream)
            assert rc == 0
            torch.cuda.synchronize()
            outs.append((sim.clone(), nbr.clone(), [t.clone() for t in dst]))
        (sim_a, nbr_a, dst_a), (sim_b, nbr_b, dst_b) = outs
        # the same kernels in the same order on the same inputs: identical bits, not merely within tolerance
        assert torch.equal(sim_a, sim_b) and torch.equal(nbr_a, nbr_b)
        for a, b in zip(dst_a, dst_b):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
        assert int(nbr_b.min()) >= 0 and int(nbr_b.max()) < M


def test_static_scratch_entry_rejects_bad_arguments(device):
    lib = ctypes.CDLL(S.library_path())
    lib.spes_expert_warmup_merge_static.restype = ctypes.c_int32
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.spes_expert_warmup_merge_static.argtypes = [i32, i32, i32, ctypes.c_float, vp, i64, i32, vp, vp, vp, vp, vp, vp]
    p = ctypes.c_void_p(0x10000)
    assert lib.spes_expert_warmup_merge_static(65, 1, 4, 0.1, p, 4096, 0, None, None, None, None, p, None) == -2   # beyond 64 experts
    assert lib.spes_expert_warmup_merge_static(8, 1, 8, 0.1, p, 4096, 0, None, None, None, None, p, None) == -1    # top_K must be < n_experts
    assert lib.spes_expert_warmup_merge_static(8, 1, 4, 0.1, p, 0, 0, None, None, None, None, p, None) == -1       # empty projection

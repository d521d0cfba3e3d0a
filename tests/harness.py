"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI, compare with the oracle."""
from __future__ import annotations

import numpy as np
import torch

import paper_2602_11543_amd as S
from paper_2602_11543_amd.layer import DeviceLayer, shape_of, to_dev  # noqa: F401

TOL = {"f32": 1e-5, "bf16": 2e-2}     # max |a-b| / max |b| per tensor (stated by the benchmark definition)


def rel_err(got, want) -> float:
    got = np.asarray(got, dtype=np.float64); want = np.asarray(want, dtype=np.float64)
    den = np.abs(want).max()
    return float(np.abs(got - want).max() / (den if den > 0 else 1.0))


def storage_ulp_excess(got, want, mag, dtype, f32_ulps=2.0):
    """How far `got` (values of the storage type) is from the fp64 result `want`, as the largest element-wise excess
    over the allowance (<= 0: within it).  The device forms such results in fp32 from operands of magnitude up to
    `mag` and rounds once: fp32 storage may differ by `f32_ulps` fp32 ulps at the magnitude of the operands (a mean
    of nearly cancelling copies is tiny against them), bf16 storage by one bf16 ulp from the rounded fp64 value --
    or by that same fp32 allowance where the result is so small that a bf16 ulp is below it."""
    got64, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    allow32 = f32_ulps * np.spacing(np.asarray(mag, dtype=np.float32)).astype(np.float64)
    err = np.abs(got64 - want)
    if dtype == "f32":
        return float((err - allow32).max())
    from spes_workloads import bf16_round

    def ordered(a):        # bf16 values as integers that count representable steps, monotone through zero
        b = np.asarray(a, dtype=np.float32).view(np.int32).astype(np.int64) >> 16
        return np.where(b < 0, -(b & 0x7FFF), b)

    steps = np.abs(ordered(got) - ordered(bf16_round(want.astype(np.float32))))
    bad = (steps > 1) & (err > 2 * allow32)
    return float(np.where(bad, steps, 0).max())


def oracle_run(inp, O, keep=True):
    cfg = inp["cfg"]
    fwd = O.moe_forward(inp["x"], inp["w_router"], inp["router_bias"], inp["w_gate"], inp["w_up"], inp["w_down"],
                        cfg.k, cfg.renorm, keep=keep)
    return fwd


def check_routing(L: DeviceLayer, fwd) -> None:
    """Integer routing results are compared bit for bit."""
    cfg = L.cfg
    assert np.array_equal(L.idx.cpu().numpy(), fwd["idx"]), "top-k indices differ"
    assert np.array_equal(L.count.cpu().numpy(), fwd["count"]), "per-expert counts differ"
    assert np.array_equal(L.view("offset").cpu().numpy(), fwd["offset"])
    assert np.array_equal(L.view("perm").cpu().numpy(), fwd["perm"]), "permutation differs"
    assert np.array_equal(L.view("inv").cpu().numpy(), fwd["inv"])
    assert int(L.count.sum()) == cfg.T * cfg.k
    # dispatch is a copy: row r of the permuted input is the input row of pair perm[r], bit for bit
    xp = L.permuted()
    want = L.x[torch.from_numpy(fwd["perm"] // cfg.k).to(L.dev).long()]
    assert torch.equal(xp.view(torch.uint8), want.contiguous().view(torch.uint8)), "permuted input differs"

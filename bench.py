#!/usr/bin/env python3
"""Benchmark of the SPES MoE-layer hot path on one MI355X.

One step = one forward plus one backward of the routed SwiGLU layer (every stage
of the hot path: router GEMM, softmax/top-k, histogram/scan/rank, dispatch, grouped
expert GEMMs, combine; backward with weight gradients for the trainable experts
only) over one batch of seeded synthetic tokens already resident in HBM.  The
dispatch copy is fused into the operand reads of the grouped GEMMs; its stand-alone
kernel (spes_moe_permute) and the stand-alone backward of the combine (spes_moe_grad_scatter) are timed beside the
step and reported with in_step false.

Without --config the headline is the largest single-GPU layer workload of the benchmark; the other layer workloads and
the expert-merge sweep are timed after it with the same step counts and reported under other_workloads.

Prints one JSON line: layer tokens/s, the roofline position of the dominant kernel
(measured with HIP events recorded between stages on the launch stream), per-stage
figures, and the fp64 CPU oracle timed on a bounded token sample as a baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak
PEAK_FP32_TFLOPS = 157.3      # fp32 vector/matrix peak (fp32 storage mode)
PEAK_HBM_GBS = 8000.0         # HBM3E


# kernel behind each single-launch stage, as named in the rocprofv3 summaries under profiles/
STAGE_KERNEL = {
    "gemm_gate_up_swiglu": "gemm_mfma_kernel<0, 1, true, true, false",
    "gemm_down": "gemm_mfma_kernel<0, 0, true, true, false",
    "gemm_dgrad_down_dswiglu": "gemm_mfma_kernel<0, 2, true, false, false",
    "gemm_dgrad_gate_up": "gemm_mfma_kernel<0, 0, true, false, false",
    "wgrad_down": "gemm_mfma_kernel<1, 0, false, false, true",
    "permute": "permute_kernel",
    "combine": "combine_kernel",
}


def profiled_traffic(cfg_name: str, stage: str):
    """HBM-side bytes per launch of the stage's kernel from the committed counter summary of this workload
    (FETCH_SIZE and WRITE_SIZE in KiB, each scaled by what the same counter reads for a plain copy of known size),
    or None when there is no summary for the workload or the stage is not a single kernel of its own."""
    path = os.path.join(ROOT, "profiles", f"moe_layer_{cfg_name}.txt")
    kernel = STAGE_KERNEL.get(stage)
    if kernel is None or not os.path.exists(path):
        return None
    fetch = write = None
    sf = sw = None
    in_table = False
    for line in open(path):
        if line.startswith("# HBM"):
            in_table = True
        elif line.startswith("# calibration"):
            in_table = False
        elif in_table and line.startswith(kernel):
            cols = line.split()
            fetch, write = float(cols[-2]), float(cols[-1])
        elif line.startswith("# scale factors:"):
            nums = [float(t.lstrip("x").rstrip(",")) for t in line.split() if t.startswith("x")]
            if len(nums) == 2:
                sf, sw = nums
    if None in (fetch, write, sf, sw):
        return None
    return {"bytes": int((fetch * sf + write * sw) * 1024), "fetch_bytes": int(fetch * sf * 1024), "write_bytes": int(write * sw * 1024),
            "source": f"profiles/moe_layer_{cfg_name}.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, calibrated on a 1 GiB copy)"}


def stage_model(cfg, rho_rows):
    """Algorithmic work of every stage: (bound, amount) with amount in FLOP (mfma/alu) or bytes (hbm)."""
    T, d, M, f, k = cfg.T, cfg.d, cfg.M, cfg.f, cfg.k
    R = T * k
    s = 4 if cfg.dtype == "f32" else 2
    mm = "alu" if cfg.dtype == "f32" else "mfma"
    return {
        "router_gemm": ("hbm", T * d * s + M * d * s + T * M * 4),
        "softmax_topk": ("hbm", T * M * 4 + 2 * R * 4 * 2 + T * 4),
        "hist_scan_rank": ("hbm", R * 4 * 7),
        "permute": ("hbm", T * d * s + R * d * s),
        "grad_scatter": ("hbm", T * d * s + 2 * R * d * s + R * 12),      # dy once, yp rows in, scaled rows out, gate/inv/dgate
        "gemm_gate_up_swiglu": (mm, 4.0 * R * d * f),
        "gemm_down": (mm, 2.0 * R * d * f),
        "combine": ("hbm", R * d * s + T * d * s + R * 8),
        "gemm_dgrad_down_dswiglu": (mm, 2.0 * R * d * f),
        "gating_bwd": ("hbm", T * M * 4 * 2 + R * 4 * 4),
        "gemm_dgrad_gate_up": (mm, 4.0 * R * d * f),
        "wgrad_down": (mm, 2.0 * rho_rows * d * f),
        "wgrad_gate": (mm, 2.0 * rho_rows * d * f),
        "wgrad_up": (mm, 2.0 * rho_rows * d * f),
        "router_wgrad": ("hbm", T * d * s + T * M * 4 + M * d * 4),
        "router_dgrad": ("hbm", T * M * 2 + M * d * s + T * d * s),          # bf16 storage only: its own small GEMM
        # sum of the k permuted gradient rows plus the router part (read as a precomputed row in bf16 storage)
        "unpermute_sum_router_dgrad": ("hbm", R * d * s + T * d * s + R * 4 + (T * d * s if s == 2 else 0)),
    }


def merge_figures(args) -> dict:
    """Expert synchronisation sweep (16 node copies of a 64-expert layer, d=2048, f=1024, bf16) and warm-up merge."""
    import numpy as np
    import torch

    import paper_2602_11543_amd as S

    dev = torch.device("cuda:0")
    M, d, f, nodes, per = 64, 2048, 1024, 16, 16
    E = d * f
    rng = np.random.default_rng(20260216)
    slot = np.full((nodes, M), -1, dtype=np.int32)
    for i in range(nodes):
        sub = np.sort(rng.permutation(M)[:per])
        slot[i, sub] = np.arange(per, dtype=np.int32)
    w = (0.5 + rng.random(nodes)).astype(np.float32)
    cnt = (slot >= 0).sum(0)
    mats = []
    for _ in range(3):   # gate, up, down projections: one call per parameter matrix
        base = (torch.randn(M, E, device=dev) * 0.02).to(torch.bfloat16)
        stores = [(torch.randn(per, E, device=dev) * 0.02).to(torch.bfloat16) for _ in range(nodes)]
        mats.append((base, stores))
    tc = torch.empty(M, dtype=torch.int32, device=dev)

    def sync_step():
        for base, stores in mats:
            S.spes_expert_merge(M, E, S.SPES_BF16, stores, slot, w, base, tc)

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(steps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / steps

    ms_sync = timed(sync_step, args.steps, args.warmup)
    bytes_sync = 3 * 2 * E * (int(cnt.sum()) + int((cnt > 0).sum()))
    # warm-up merge on the merged store: similarity on the gate projection, all three matrices mixed
    K, alpha = 4, 0.1
    srcs = [m[0] for m in mats]
    dsts = [torch.empty_like(t) for t in srcs]
    sim = torch.empty(M, M, dtype=torch.float32, device=dev)
    nbr = torch.empty(M, K, dtype=torch.int32, device=dev)
    scratch = torch.empty(S.spes_warmup_scratch_bytes(M, E), dtype=torch.uint8, device=dev)

    def warm_step():
        S.spes_expert_warmup_merge(M, S.SPES_BF16, K, alpha, srcs[0], E, srcs, dsts, [E, E, E], sim, nbr, scratch)

    ms_warm = timed(warm_step, args.steps, args.warmup)
    # similarity and peer selection alone (no matrix to mix): one pass over the input projections
    ms_gram = timed(lambda: S.spes_expert_warmup_merge(M, S.SPES_BF16, K, alpha, srcs[0], E, [], [], [], sim, nbr, scratch),
                    args.steps, args.warmup)
    bytes_warm = 2 * M * E + 3 * 2 * M * E * (K + 1 + 1)      # Gram pass + (K+1) reads and one write per matrix
    bytes_warm_once = 2 * M * E + 3 * 2 * M * E * 2           # every matrix read once and written once (peer re-reads from cache)
    out = {"metric": "expert merge GB/s on 1 MI355X", "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"cfg5 merge: {nodes} nodes x {per} of {M} experts, d={d} f={f}, 3 matrices, weighted; "
                                  f"trainers/expert min {int(cnt.min())} max {int(cnt.max())} sum {int(cnt.sum())}"},
           "sync_merge": {"ms": round(ms_sync, 4), "bytes": bytes_sync, "achieved": round(bytes_sync / ms_sync / 1e6, 1),
                          "peak": PEAK_HBM_GBS, "frac": round(bytes_sync / ms_sync / 1e6 / PEAK_HBM_GBS, 4), "bound": "hbm"},
           # priced on the bytes that must move (every matrix read once and written once, the similarity input read once);
           # the K peer reads per element are requests that the L2 serves
           "warmup_merge": {"ms": round(ms_warm, 4), "bytes": bytes_warm_once, "achieved": round(bytes_warm_once / ms_warm / 1e6, 1),
                            "peak": PEAK_HBM_GBS, "frac": round(bytes_warm_once / ms_warm / 1e6 / PEAK_HBM_GBS, 4), "bound": "hbm",
                            "K": K, "alpha": alpha,
                            "similarity_pass": {"ms": round(ms_gram, 4), "bytes": 2 * M * E, "bound": "hbm",
                                                "achieved": round(2 * M * E / ms_gram / 1e6, 1), "peak": PEAK_HBM_GBS,
                                                "frac": round(2 * M * E / ms_gram / 1e6 / PEAK_HBM_GBS, 4)},
                            "requested_bytes": bytes_warm,
                            "requested_rate": round(bytes_warm / ms_warm / 1e6, 1)}}
    out["value"] = out["sync_merge"]["achieved"]
    del mats, srcs, dsts, scratch
    torch.cuda.empty_cache()
    return out


def bench_merge(args) -> int:
    print(json.dumps(merge_figures(args)))
    return 0


def bench_train_step(args) -> int:
    """One node's whole update of the layer: forward, auxiliary router losses, backward, AdamW on the trainable experts
    and the router (the headline workload plus the two neighbouring stages, timed separately)."""
    import numpy as np
    import torch

    import paper_2602_11543_amd as S
    from spes_workloads import CONFIGS, layer_inputs
    from paper_2602_11543_amd.layer import DeviceLayer

    cfg = CONFIGS[args.config]
    dev = torch.device("cuda:0")
    L = DeviceLayer(layer_inputs(cfg), dev)
    n, M, d, f = len(L.trainable), cfg.M, cfg.d, cfg.f
    dt = S.SPES_F32 if cfg.dtype == "f32" else S.SPES_BF16
    hyper = dict(lr=5e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    state = []
    for w, g, elems in ((L.w_gate, L.d_w_gate, f * d), (L.w_up, L.d_w_up, f * d), (L.w_down, L.d_w_down, d * f)):
        master = w[L.trainable].float().reshape(n, elems).contiguous()
        state.append((w, L.mask, master, torch.zeros_like(master), torch.zeros_like(master), g, M, elems))
    rmaster = L.w_router.float().reshape(1, M * d).contiguous()
    state.append((L.w_router, np.ones(1, dtype=np.uint8), rmaster, torch.zeros_like(rmaster), torch.zeros_like(rmaster),
                  L.d_w_router, 1, M * d))
    losses = torch.zeros(2, dtype=torch.float32, device=dev)
    step_no = [0]

    def optim():
        step_no[0] += 1
        for w, mask, master, m, v, g, ne, elems in state:
            S.spes_masked_adamw(ne, elems, dt, w, mask, master, m, v, g, step=step_no[0], **hyper)

    def aux():
        S.spes_moe_router_aux(L.shape, L.ctx, 0.01, 0.001, 1.0, losses)

    def timed(parts, steps, warmup):
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(parts) + 1)] for _ in range(steps)]
        for _ in range(warmup):
            for fn in parts:
                fn()
        torch.cuda.synchronize()
        for i in range(steps):
            ev[i][0].record()
            for j, fn in enumerate(parts):
                fn()
                ev[i][j + 1].record()
        torch.cuda.synchronize()
        return [sum(ev[i][j].elapsed_time(ev[i][j + 1]) for i in range(steps)) / steps for j in range(len(parts))]

    t_fwd, t_aux, t_bwd, t_opt = timed([L.fwd, aux, L.bwd, optim], args.steps, args.warmup)
    total = t_fwd + t_aux + t_bwd + t_opt
    es = 4 if cfg.dtype == "f32" else 2
    opt_elems = 3 * n * d * f + M * d
    opt_bytes = opt_elems * (28 + es)          # grad, m, v, w in; m, v, w out; the storage-type copy out
    aux_bytes = cfg.T * M * 4 + cfg.T * 4      # scores and log-sum-exp read once
    out = {"metric": "MoE layer training step (fwd + aux losses + bwd + AdamW on the trainable subset) tokens/sec on 1 MI355X",
           "value": round(cfg.T / total * 1e3, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(total, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
           "config": {"workload": f"{cfg.name}: T={cfg.T} d_model={cfg.d} experts={M} d_ff={f} top_k={cfg.k} trainable={n}/{M}"},
           "stages": {"fwd": {"ms": round(t_fwd, 4)}, "bwd": {"ms": round(t_bwd, 4)},
                      "router_aux": {"ms": round(t_aux, 4), "bound": "hbm", "achieved": round(aux_bytes / t_aux / 1e6, 1),
                                     "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(aux_bytes / t_aux / 1e6 / PEAK_HBM_GBS, 4)},
                      "masked_adamw": {"ms": round(t_opt, 4), "bound": "hbm", "bytes": opt_bytes,
                                       "achieved": round(opt_bytes / t_opt / 1e6, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                       "frac": round(opt_bytes / t_opt / 1e6 / PEAK_HBM_GBS, 4)}},
           "losses": {"load_balancing": float(losses[0]), "router_z": float(losses[1])}}
    print(json.dumps(out))
    return 0


def bench_init(args) -> int:
    """Upcycling initialiser and upload packing on the upcycled workload's shape (32 experts of 4864 x 3584, bf16)."""
    import numpy as np
    import torch

    import paper_2602_11543_amd as S

    dev = torch.device("cuda:0")
    M, elems, n_tr = 32, 4864 * 3584, 8
    dense = (torch.randn(elems, device=dev) * 0.02).to(torch.bfloat16)
    out = torch.empty(M, elems, dtype=torch.bfloat16, device=dev)
    mask = np.zeros(M, dtype=np.uint8); mask[np.random.default_rng(0).choice(M, n_tr, replace=False)] = 1
    packed = torch.empty(n_tr, elems, dtype=torch.bfloat16, device=dev)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(args.steps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / args.steps

    ms_up = timed(lambda: S.spes_upcycle_init(M, elems, S.SPES_BF16, dense, 0.5, 0.02, 7, 1, out))
    ms_pk = timed(lambda: S.spes_expert_pack(M, elems, S.SPES_BF16, out, mask, packed, 0))
    by_up = 2 * elems * (M + 1)                 # every expert written once; the dense matrix read (cache-served after the first)
    by_pk = 2 * 2 * elems * n_tr
    res = lambda ms, by: {"ms": round(ms, 4), "bytes": by, "bound": "hbm", "achieved": round(by / ms / 1e6, 1), "peak": PEAK_HBM_GBS,
                          "unit": "GB/s", "frac": round(by / ms / 1e6 / PEAK_HBM_GBS, 4)}
    out_j = {"metric": "upcycling initialiser GB/s on 1 MI355X", "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
             "warmup": args.warmup, "dtype": "bf16", "data": "synthetic",
             "config": {"workload": f"{M} experts x {elems} elements from one dense matrix, noise on 50 %; pack of {n_tr} experts"},
             "upcycle_init": res(ms_up, by_up), "expert_pack": res(ms_pk, by_pk)}
    # the initialiser is bound by the generator's 64-bit integer multiplies, not by memory: no roofline claim
    out_j["upcycle_init"].update(bound="alu", peak=None, frac=None)
    out_j["value"] = out_j["upcycle_init"]["achieved"]
    print(json.dumps(out_j))
    return 0


def layer_figures(cfg_name: str, args, full: bool) -> dict:
    """Times fwd + bwd of the layer workload `cfg_name`.  full: also the per-stage breakdown, the stand-alone dispatch and
    gradient-scatter kernels, the matrix-rate reference and the CPU oracle; otherwise step time and stage durations only."""
    import numpy as np
    import torch

    import paper_2602_11543_amd as S
    from paper_2602_11543_amd.layer import DeviceLayer
    from spes_workloads import CONFIGS, layer_inputs

    dev = torch.device("cuda:0")
    cfg = CONFIGS[cfg_name]
    t0 = time.time()
    inp = layer_inputs(cfg)
    L = DeviceLayer(inp, dev)
    gen_s = time.time() - t0

    def step():
        L.fwd()
        L.bwd(0)

    copy_gbs = fill_gbs = None
    if full:
        # a plain 1 GiB device copy: reference point for the HBM byte counters and for what a stream achieves here
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            dst.copy_(src)              # reads 1 GiB, writes 1 GiB
        e1.record()
        torch.cuda.synchronize()
        copy_gbs = 3 * 2 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9
        # a pure write stream (the dispatch copy is eight ninths writes at top-8)
        e0.record()
        for _ in range(3):
            dst.fill_(7)
        e1.record()
        torch.cuda.synchronize()
        fill_gbs = 3 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del src, dst

    run = step
    if args.graph:
        # the step recorded once into a HIP graph and replayed: removes the host's per-kernel launch cost (measured: no
        # difference even on the smallest workload, whose time is the latency of its dependent small kernels)
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            step()
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.synchronize()
        run = graph.replay
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    tokens_per_s = cfg.T / (ms_per_step * 1e-3)

    # per-stage durations: HIP events recorded by the library on the launch stream, averaged over the same number of steps
    S.spes_profile_enable(True)
    acc = {}
    for _ in range(args.steps):
        L.fwd()
        f_st = S.spes_profile_read(0)
        L.bwd(0)
        b_st = S.spes_profile_read(1)
        for n, ms in f_st + b_st:
            acc[n] = acc.get(n, 0.0) + ms
    S.spes_profile_enable(False)
    stage_ms = {n: v / args.steps for n, v in acc.items()}
    standalone = {}
    if full:
        # the dispatch copy and the gradient scatter are not part of the step (the grouped GEMMs read x and dy through the
        # routing table); their stand-alone kernels are timed here on the same stream, from the record the last forward left
        def timed_alone(fn):
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            fn()
            ev[0].record()
            for _ in range(args.steps):
                fn()
            ev[1].record()
            torch.cuda.synchronize()
            return ev[0].elapsed_time(ev[1]) / args.steps
        xp = torch.empty(cfg.T * cfg.k, cfg.d, dtype=L.x.dtype, device=dev)
        dgate = torch.empty(cfg.T, cfg.k, dtype=torch.float32, device=dev)
        standalone["permute"] = timed_alone(lambda: S.spes_moe_permute(L.shape, L.x, L.ctx, xp))
        standalone["grad_scatter"] = timed_alone(lambda: S.spes_moe_grad_scatter(L.shape, L.dy, L.ctx, xp, dgate))
        del xp, dgate

    # what the matrix cores reach on this device with operand values like the workload's (the shader clock under
    # matrix load is power-limited and depends on the data): a register-resident MFMA loop, no memory traffic at all;
    # run after everything that is timed, so that it does not eat into their power budget
    mfma_tflops = None
    if full and cfg.dtype == "bf16":
        sink = torch.empty(256, dtype=torch.float32, device=dev)
        S.spes_ref_mfma_rate(L.w_gate, 256, 4000, sink)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flop = sum(S.spes_ref_mfma_rate(L.w_gate, 256, 20000, sink) for _ in range(3))
        e1.record()
        torch.cuda.synchronize()
        mfma_tflops = flop / (e0.elapsed_time(e1) * 1e-3) / 1e12

    count = L.count.cpu().numpy()
    rows_trainable = int(count[np.nonzero(L.mask)[0]].sum())
    model = stage_model(cfg, rows_trainable)
    stages = {}
    for n, ms in list(stage_ms.items()) + list(standalone.items()):
        bound, amount = model[n]
        if bound == "hbm":
            ach, peak, unit = amount / (ms * 1e-3) / 1e9, PEAK_HBM_GBS, "GB/s"
        else:
            ach, unit = amount / (ms * 1e-3) / 1e12, "TFLOP/s"
            peak = PEAK_BF16_TFLOPS if bound == "mfma" else PEAK_FP32_TFLOPS
        stages[n] = dict(ms=round(ms, 4), bound=bound, achieved=round(ach, 2), peak=peak, unit=unit, frac=round(ach / peak, 4))
        if n in standalone:
            stages[n]["in_step"] = False       # timed on its own: the step does not run it
    dominant = max(stage_ms, key=stage_ms.get)
    dom = stages[dominant]
    gemm_names = [n for n, (b, _) in model.items() if b in ("mfma", "alu") and n in stage_ms]
    gemm_flop = sum(model[n][1] for n in gemm_names)
    gemm_ms = sum(stage_ms[n] for n in gemm_names)
    gemm_peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_FP32_TFLOPS

    out = {
        "metric": "MoE layer fwd+bwd tokens/sec on 1 MI355X; grouped-GEMM MFMA util %",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} d_model={cfg.d} experts={cfg.M} d_ff={cfg.f} top_k={cfg.k} "
                               f"renorm={cfg.renorm} trainable={cfg.n_trainable}/{cfg.M} ({cfg.dtype}, fp32 accumulate)",
                   "trainable_row_fraction": round(rows_trainable / (cfg.T * cfg.k), 4),
                   "max_over_mean_expert_load": round(float(count.max() / count.mean()), 2),
                   "input_generation_s": round(gen_s, 1), "hip_graph": bool(args.graph)},
        "roofline": {"kernel": dominant, "bound": dom["bound"], "achieved": dom["achieved"], "peak": dom["peak"],
                     "unit": dom["unit"], "frac": dom["frac"], "traffic": None},
        "grouped_gemm_util": {"flop": gemm_flop, "ms": round(gemm_ms, 4), "achieved_tflops": round(gemm_flop / (gemm_ms * 1e-3) / 1e12, 2),
                              "peak_tflops": gemm_peak, "frac": round(gemm_flop / (gemm_ms * 1e-3) / 1e12 / gemm_peak, 4)},
        "stages": stages,
    }
    if copy_gbs is not None:
        out["hbm_copy_reference"] = {"achieved": round(copy_gbs, 1), "unit": "GB/s", "frac": round(copy_gbs / PEAK_HBM_GBS, 4),
                                     "what": "plain 1 GiB device-to-device copy (read + write bytes) on this GPU"}
        out["hbm_fill_reference"] = {"achieved": round(fill_gbs, 1), "unit": "GB/s", "frac": round(fill_gbs / PEAK_HBM_GBS, 4),
                                     "what": "plain 1 GiB device fill (write bytes only) on this GPU"}
    if mfma_tflops is not None:
        out["mfma_reference"] = {"achieved": round(mfma_tflops, 1), "unit": "TFLOP/s", "frac_of_nominal": round(mfma_tflops / PEAK_BF16_TFLOPS, 4),
                                 "what": "register-resident 16x16x32 bf16 MFMA loop on this GPU, operands taken from the workload's expert "
                                         "weights: the power-limited matrix rate on data like the workload's"}
        out["grouped_gemm_util"]["frac_of_mfma_reference"] = round(gemm_flop / (gemm_ms * 1e-3) / 1e12 / mfma_tflops, 4)
    tr = profiled_traffic(cfg.name, dominant)
    if tr is not None:
        out["roofline"]["traffic"] = tr["bytes"]           # HBM-side bytes per launch (offline counters, see traffic_detail)
        out["roofline"]["traffic_detail"] = tr

    if full and args.cpu_sample > 0:
        from oracle import spes_oracle as O
        n = min(args.cpu_sample, cfg.T)
        xs, dys = inp["x"][:n], inp["dy"][:n]
        t0 = time.perf_counter()
        fwd = O.moe_forward(xs, inp["w_router"], inp["router_bias"], inp["w_gate"], inp["w_up"], inp["w_down"], cfg.k, cfg.renorm)
        O.moe_backward(fwd, dys, xs, inp["w_router"], inp["w_gate"], inp["w_up"], inp["w_down"], cfg.renorm,
                       wgrad_experts=L.trainable)
        cpu_s = time.perf_counter() - t0
        del fwd
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        out["cpu_baseline"] = {"value": round(n / cpu_s, 1), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
                               "sample": f"fwd+bwd of the first {n} of the workload's {cfg.T} tokens through the fp64 numpy oracle "
                                         f"(all {cfg.M} experts' weights, weight grads for the trainable ones), {cpu_s:.1f} s"}
    del L, inp
    torch.cuda.empty_cache()
    return out


HEADLINE = "cfg3"          # the largest of the benchmark's single-GPU layer workloads
ALSO = ("cfg2", "cfg4", "cfg1")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default=None,
                    help=f"workload name from spes_workloads.CONFIGS; default: {HEADLINE} as the headline, and the other "
                         f"benchmark workloads ({', '.join(ALSO)}, the cfg5 merge sweep) timed after it under `other_workloads`")
    ap.add_argument("--workload", default="layer", choices=["layer", "merge", "step", "init"],
                    help="layer: fwd+bwd of the MoE layer (the headline metric); merge: expert synchronisation sweep; "
                         "step: fwd + auxiliary losses + bwd + AdamW on the trainable subset; init: upcycling initialiser and upload packing")
    ap.add_argument("--cpu-sample", type=int, default=6144, help="tokens of the workload timed through the fp64 oracle (0: skip)")
    ap.add_argument("--graph", action="store_true", help="layer workload: replay the step from a captured HIP graph")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    if args.workload == "merge":
        return bench_merge(args)
    if args.workload == "step":
        args.config = args.config or "cfg2"
        return bench_train_step(args)
    if args.workload == "init":
        return bench_init(args)

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    out = layer_figures(args.config or HEADLINE, args, full=True)
    if args.config is None:
        # every other workload of the benchmark, timed in the same run with the same step counts
        others = {}
        for name in ALSO:
            o = layer_figures(name, args, full=False)
            others[name] = {"workload": o["config"]["workload"], "tokens_per_s": o["value"], "ms_per_step": o["ms_per_step"],
                            "dtype": o["dtype"], "grouped_gemm_util": o["grouped_gemm_util"],
                            "roofline": {k: o["roofline"][k] for k in ("kernel", "bound", "achieved", "peak", "unit", "frac")},
                            "stage_ms": {n: v["ms"] for n, v in o["stages"].items()}}
        m = merge_figures(args)
        others["cfg5_merge"] = {"workload": m["config"]["workload"], "sync_merge": m["sync_merge"], "warmup_merge": m["warmup_merge"]}
        out["other_workloads"] = others
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())

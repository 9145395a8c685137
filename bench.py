#!/usr/bin/env python3
"""Throughput of the stage-compute hot path on one MI355X.

A step is one pass of the whole hot path over one micro-batch of synthetic input that is
already resident in HBM: stage forward (saving activations) + stage backward, preceded by
the extra no-grad forward for the self-conditioned DiT workload; for the text-encoder
workload a step covers the 64-sample global batch with partial-batch calls.
`value` is the mean over exactly --steps steps between two device synchronisations (wall clock); the median of the
per-step times taken with events on the launch stream is reported beside it.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_PEAK = 2.5e15      # MI355X dense bf16 MFMA, FLOP/s
HBM_PEAK = 8.0e12       # B/s


def stage_flops(cfg):
    """Algorithmic FLOPs of one step (2mnk per GEMM; backward = 2x forward except the context
    K/V projection (weight gradient only); attention backward = 2x forward; no credit for
    recomputation or padding)."""
    B, N, d, H, dh = cfg.batch, cfg.tokens, cfg.d_model, cfg.n_heads, cfg.d_head
    T = B * N
    if cfg.kind == "unet_xattn_geglu":
        Lc, dc, inner = cfg.ctx_tokens, cfg.ctx_dim, cfg.ff_inner
        gemm = 2 * T * d * 3 * d + 2 * T * d * d            # qkv, out
        gemm += 2 * T * d * d * 2                             # cross q, out
        gemm += 2 * T * d * 2 * inner + 2 * T * inner * d     # ff
        kv = 2 * B * Lc * dc * 2 * d
        attn = 4 * B * H * N * N * dh + 4 * B * H * N * Lc * dh
        fwd = gemm + kv + attn
        bwd = 2 * gemm + kv + 2 * attn
    else:
        ff = cfg.ff_inner
        gemm = 2 * T * d * 3 * d + 2 * T * d * d + 2 * T * d * ff * 2 + 2 * B * d * 6 * d
        attn = 4 * B * H * N * N * dh
        fwd = gemm + attn
        bwd = 2 * (gemm + attn)
    total = (fwd + bwd) * cfg.n_blocks
    if cfg.self_cond:
        total += fwd * cfg.n_blocks
    return float(total)


def encoder_flops_per_sample(c):
    d, ff, S = c.d_model, c.ff_inner, c.seq
    per_layer = 2 * S * d * 3 * d + 2 * S * d * d + 2 * S * d * ff * 2 + 4 * c.n_heads * S * S * c.d_head
    return float(per_layer * c.n_layers)


def image_encoder_flops_per_sample(c):
    """2 * pixels * c_out * 9 c_in per 3x3 convolution, 2mnk per 1x1 convolution, 4 * pixels^2 * c for the attention block."""
    h, w, fl = c.height, c.width, 0.0
    for (kind, ci, co, st) in c.layers:
        px = h * w
        if kind == "conv":
            h, w = (h - 1) // st + 1, (w - 1) // st + 1
            fl += 2.0 * h * w * co * 9 * ci
        elif kind == "resnet":
            fl += 2.0 * px * co * 9 * ci + 2.0 * px * co * 9 * co + (2.0 * px * co * ci if ci != co else 0.0)
        elif kind == "attn":
            fl += 4 * 2.0 * px * ci * ci + 4.0 * px * px * ci
        else:
            fl += 2.0 * px * co * 9 * ci
    return fl


def timed(fn, steps, warmup, median_out=None):
    """Mean wall-clock seconds per step over exactly `steps` steps between two device synchronisations.  The same steps
    are bracketed one by one with events on the stream the work is launched on; median_out["ms"] receives their median."""
    import torch
    for _ in range(warmup):
        fn()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / steps
    if median_out is not None:
        per = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
        median_out["ms"] = per[len(per) // 2] if steps % 2 else 0.5 * (per[steps // 2 - 1] + per[steps // 2])
    return sec


def cpu_baseline_stage(cfg):
    """The fp64 oracle as it stands, timed on a bounded sample (a few samples of the workload)."""
    import synth_inputs as si
    from oracle import blocks
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1

    def run(nb):
        c = cfg.replace(batch=nb)
        inp = si.make_stage_inputs(c, seed=0)
        cc = inp["ctx"] if c.kind == si.UNET else inp["cond"]
        t0 = time.perf_counter()
        if c.self_cond:
            blocks.stage_self_conditioned(c.kind, inp["params"], inp["x_sc"], inp["x"], cc, inp["dy"], c.n_blocks, c.n_heads,
                                          c.ln_eps, bool(c.gelu_tanh))
        else:
            _, caches = blocks.stage_fwd(c.kind, inp["params"], inp["x"], cc, c.n_blocks, c.n_heads, c.ln_eps, bool(c.gelu_tanh))
            blocks.stage_bwd(c.kind, inp["params"], caches, inp["dy"], c.n_heads)
        return time.perf_counter() - t0

    t1 = run(1)
    nb, t = 1, t1
    if t1 < 6.0 and cfg.batch > 1:
        nb = int(min(cfg.batch, max(2, 12.0 // max(t1, 1e-3))))
        t = run(nb)
    return {"value": nb / t, "unit": "samples/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{nb} of {cfg.batch} samples of {cfg.name}, one fp64 numpy fwd+bwd"
                      + (" incl. the extra no-grad forward" if cfg.self_cond else "") + f", {t:.1f} s"}


def cpu_baseline_image_encoder(cfg):
    """The fp64 oracle of the image encoder on one sample of the workload (about half a minute)."""
    import synth_inputs as si
    from oracle import image_encoder as ie
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    c = cfg.replace(global_batch=1)
    inp = si.make_image_encoder_inputs(c, seed=0, weight_std=0.0)
    t0 = time.perf_counter()
    ie.encoder_fwd(inp["params"], c.layer_dicts(), inp["x"], c.groups, c.gn_eps)
    t = time.perf_counter() - t0
    return {"value": 1.0 / t, "unit": "samples/s", "cores": int(cores), "kind": "oracle",
            "sample": f"1 of {cfg.global_batch} samples of {cfg.name}, one fp64 numpy forward, {t:.1f} s"}


def pmc_traffic_bytes(workload, kind):
    """HBM bytes per launch of a kernel class as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (two counter runs,
    scaled by kernels of known size): read from the class table of profiles/hbm_traffic_<workload>.md, which also holds the
    commands.  None (with the reason) when that summary or that class is not there."""
    import re
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.md")
    if not os.path.exists(path):
        return None, f"profiles/hbm_traffic_{workload}.md is missing"
    for line in open(path):
        m = re.match(r"\|\s*`class:([a-z0-9_]+)`\s*\|\s*(\d+)\s*\|\s*([0-9.]+)\s*\|", line)
        if m and m.group(1) == kind:
            return float(m.group(3)) * 1e6, f"profiles/hbm_traffic_{workload}.md, class {kind}, {m.group(2)} dispatches"
    return None, f"profiles/hbm_traffic_{workload}.md has no row for class {kind}"


MFMA_KINDS = {"gemm_nt", "gemm_nn", "gemm_tn", "attn_fwd", "attn_bwd_dq", "attn_bwd_dkv", "conv3x3"}
KERNEL_NAMES = {"gemm_nt": "dp::gemm_bf16_dtl_kernel<..., A_MC=false, B_MC=false> (y = x W^T; dx = dy W on transposed weight copies)",
                "gemm_nn": "dp::gemm_bf16_kernel<..., A_MC=false, B_MC=true> (dx = dy W)",
                "gemm_tn": "dp::gemm_bf16_kernel<..., A_MC=true, B_MC=true> (dW = dy^T x)",
                "attn_fwd": "dp::attn_fwd_bf16_kernel", "attn_bwd_dq": "dp::attn_bwd_dq_bf16_kernel",
                "attn_bwd_dkv": "dp::attn_bwd_dkv_bf16_kernel", "ln_fwd": "dp::ln_fwd_kernel", "ln_bwd": "dp::ln_bwd_kernel",
                "geglu_fwd": "dp::geglu_fwd_kernel", "geglu_bwd": "dp::geglu_bwd_kernel", "reduce": "dp::colsum_kernel",
                "conv3x3": "dp::conv3x3_bf16_kernel (implicit GEMM)", "groupnorm": "dp::gn_partial_kernel + gn_finalize_kernel + gn_apply_kernel",
                "softmax_rows": "dp::softmax_rows_kernel"}


def kernel_roofline(workload, names, si, DeviceStage, DeviceEncoder, passes=3):
    import torch
    from paper_2405_01248_amd import binding
    if workload == "cfg5":
        obj = DeviceEncoder(si.CONFIG5, si.make_encoder_inputs(si.CONFIG5, seed=0))
        run = lambda: obj.run_slices(si.CONFIG5.global_batch)
    elif workload == "cfg6":
        from paper_2405_01248_amd.harness import DeviceImageEncoder
        obj = DeviceImageEncoder(si.CONFIG6, si.make_image_encoder_inputs(si.CONFIG6, seed=0, weight_std=0.0))
        run = lambda: obj.run_slices(si.CONFIG6.global_batch)
    else:
        obj = DeviceStage(names[workload], si.make_stage_inputs(names[workload], seed=0))
        # single-kernel durations: issue the backward's side-stream work in program order
        obj.stage.set_overlap(False)
        run = obj.step
    run()
    torch.cuda.synchronize()
    binding.ktime_begin()
    for _ in range(passes):
        run()
    recs = binding.ktime_end()
    event_overhead_us = 1e3 * binding.ktime_event_overhead_ms()
    agg = {}
    for r in recs:
        a = agg.setdefault(r["kind"], {"launches": 0, "ms": 0.0, "flops": 0.0, "bytes": 0.0})
        a["launches"] += 1; a["ms"] += r["ms"]; a["flops"] += r["flops"]; a["bytes"] += r["bytes"]
    total = sum(a["ms"] for a in agg.values())
    classes = {}
    for k, a in sorted(agg.items(), key=lambda kv: -kv[1]["ms"]):
        c = {"launches_per_step": a["launches"] / passes, "ms_per_step": a["ms"] / passes, "share": a["ms"] / total,
             "avg_launch_us": 1e3 * a["ms"] / a["launches"]}
        if k in MFMA_KINDS:
            c["tflops"] = a["flops"] / (a["ms"] * 1e-3) / 1e12
        else:
            c["gbps"] = a["bytes"] / (a["ms"] * 1e-3) / 1e9
        classes[k] = c
    dom = max(agg, key=lambda k: agg[k]["ms"])
    a = agg[dom]
    if dom in MFMA_KINDS:
        ach = a["flops"] / (a["ms"] * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": ach, "peak": MFMA_PEAK / 1e12, "unit": "TFLOP/s", "frac": ach / (MFMA_PEAK / 1e12)}
    else:
        ach = a["bytes"] / (a["ms"] * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": ach / (HBM_PEAK / 1e9)}
    traffic, traffic_src = pmc_traffic_bytes(workload, dom)
    roof.update(traffic=traffic, traffic_source=traffic_src, kernel=KERNEL_NAMES.get(dom, dom),
                note="durations from a pass with the backward's side stream disabled (kernels run one at a time); "
                     "HIP events around every launch, dispatch gap included (rocprofv3's kernel-only averages are in "
                     f"profiles/kernels_{workload}_serial.md; an empty event pair reads event_pair_overhead_us)",
                event_pair_overhead_us=event_overhead_us,
                avg_launch_us=1e3 * a["ms"] / a["launches"], launches_per_step=a["launches"] / passes,
                algorithmic_per_launch=(a["flops"] if dom in MFMA_KINDS else a["bytes"]) / a["launches"],
                # what `traffic` compares with: operands, result and every tensor the fused epilogue reads or writes, once
                tensor_bytes_per_launch=a["bytes"] / a["launches"])
    del obj
    return roof, classes


def fp8_report():
    """The FP8 (OCP E4M3) projection GEMM beside the bf16 one on the projection shapes of the DiT stage, the text encoder
    at 16 and 64 samples and one large square problem: microseconds per launch (events on the launch stream) and
    algorithmic TFLOP/s; the fp8 figure is against the 5.0 PFLOP/s fp8 peak."""
    import torch
    from paper_2405_01248_amd import binding as B
    dev = "cuda:0"

    def t(f, iters=30):
        for _ in range(3):
            f()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters * 1e3

    rows = []
    for (M, N, K) in [(8192, 4608, 1152), (8192, 1152, 4608), (8192, 3456, 1152), (4928, 3072, 768), (1232, 3072, 768), (8192, 8192, 8192)]:
        A = torch.randn((M, K), device=dev, dtype=torch.bfloat16)
        W = torch.randn((N, K), device=dev, dtype=torch.bfloat16) * 0.05
        Cc = torch.empty((M, N), device=dev, dtype=torch.bfloat16)
        ws = torch.empty(max(B.op_gemm_workspace_bytes(M, N, K), 256), dtype=torch.uint8, device=dev)
        qa = torch.zeros((M, K), dtype=torch.uint8, device=dev)
        qw = torch.zeros((N, K), dtype=torch.uint8, device=dev)
        sa, sw = float(A.abs().max()) / 448.0, float(W.abs().max()) / 448.0
        B.op_quantize_fp8(A, K, qa, K, M, K, sa)
        B.op_quantize_fp8(W, K, qw, K, N, K, sw)
        us16 = t(lambda: B.op_gemm(B.DP_BF16, A, K, 0, W, K, 0, M, N, K, None, Cc, N, False, False, ws, 0))
        us8 = t(lambda: B.op_gemm_fp8(qa, K, qw, K, M, N, K, sa * sw, None, Cc, N))
        usq = t(lambda: B.op_quantize_fp8(A, K, qa, K, M, K, sa))
        fl = 2.0 * M * N * K
        rows.append({"M": M, "N": N, "K": K, "bf16_us": us16, "bf16_tflops": fl / us16 / 1e6, "fp8_us": us8, "fp8_tflops": fl / us8 / 1e6,
                     "fp8_peak_frac": fl / us8 / 1e6 / 5000.0, "speedup": us16 / us8, "quantize_activations_us": usq})
    return {"metric": "fp8_vs_bf16_projection_gemm", "dtype": "fp8_e4m3", "shapes": rows}


def partition_report(si, DeviceStage):
    """Partitioner (Sec. 4.1 / 4.3) on cost rows measured here: the 7 identical-shape DiT blocks of cfg4 are profiled at
    local batch 32 / r for r = 1, 2, 4, 8 and tiled 4x to the 28 layers of the whole backbone; link figures are one xGMI
    link for p2p and a 7-link reduce-scatter + all-gather for the gradient all-reduce."""
    import torch
    from paper_2405_01248_amd import binding
    from oracle import partition as P      # timed beside the library as the CPU baseline of this row
    base = si.CONFIG4
    rows = []
    for b in (32, 16, 8, 4):
        cfg = base.replace(batch=b, name=f"{base.name}_b{b}")
        ds = DeviceStage(cfg, si.make_stage_inputs(cfg, seed=0))
        ds.step()
        blk = ds.stage.profile(ds.params, ds.x, ds.cc, ds.y, ds.dy, ds.dx, ds.d_cond, ds.dparams, ds.ws, reps=10)
        torch.cuda.synchronize()
        for rep in range(4):
            rows += [dict(r, layer=r["layer"] + rep * cfg.n_blocks) for r in blk]
        del ds
        torch.cuda.empty_cache()
    L = 4 * base.n_blocks
    prof = P.Profile(L, {}, {}, {}, {}, [0] * L, {})
    for r in rows:
        for name, tab in (("fwd_ms", prof.fwd_ms), ("bwd_ms", prof.bwd_ms), ("cf_bytes", prof.cf_bytes), ("cb_bytes", prof.cb_bytes)):
            tab.setdefault(r["batch"], [0] * L)[r["layer"]] = r[name]
        prof.grad_bytes[r["layer"]] = r["grad_bytes"]
        if r["layer"] == L - 1:
            prof.out_bytes[r["batch"]] = r["out_bytes"]
    link = dict(p2p_gbps=153.0, p2p_latency_ms=0.01, ar_gbps=7 * 153.0 / 2, ar_latency_ms=0.05)
    out = {"workload": "cfg4 blocks tiled to 28 layers, B=32, M=8, D=8", "links": link,
           "per_layer_ms": {str(b): {"fwd": prof.fwd_ms[b][0], "bwd": prof.bwd_ms[b][0]} for b in sorted(prof.fwd_ms)}, "plans": []}
    for p, uni in ((0.0, False), (0.5, False), (0.5, True)):
        t0 = time.perf_counter()
        for _ in range(20):
            got = binding.partition_solve(rows, 32, 8, 8, self_cond_prob=p, uniform_replication=uni, **link)
        t_lib = (time.perf_counter() - t0) / 20
        o = P.Options(micro_batch=32, n_micro_batches=8, n_devices=8, self_cond_prob=p, uniform_replication=uni, **link)
        t0 = time.perf_counter()
        ref = P.solve(prof, o)
        t_or = time.perf_counter() - t0
        same = (got["first_layer"], got["replicas"]) == (ref.first_layer, ref.replicas) and abs(got["t_max_ms"] - ref.t_max_ms) <= 1e-9 * ref.t_max_ms
        out["plans"].append({"self_cond_prob": p, "uniform_replication": uni, "layers_per_stage": got["n_layers"], "replicas": got["replicas"],
                             "t0_ms": got["t0_ms"], "gap_ms": got["gap_ms"], "t_max_ms": got["t_max_ms"], "solve_ms_library": t_lib * 1e3,
                             "solve_ms_oracle": t_or * 1e3, "matches_oracle": same})
    return out, prof, rows


def bidirectional_report(si, DeviceStage):
    """Bidirectional partitioning of two backbones (Sec. 4.2, Eq. 10-16) on cost rows measured here: the U-Net blocks of
    cfg2 (32x32 latents, d = 640) as the backbone pipelined down the device chain and those of cfg3 (64x64 latents,
    d = 320) as the one pipelined up, each profiled at local batch 8 / 4 / 2 and tiled to 6 layers; 4 devices, micro-batch
    8, M_CDM = 8 (an input: the paper prints no expression for it), one xGMI link for p2p, 7 links for the all-reduce."""
    import torch
    from paper_2405_01248_amd import binding
    from oracle import partition as P      # timed beside the library as the CPU baseline of this row
    tiles, profs, all_rows = 3, [], []
    for base in (si.CONFIG2, si.CONFIG3):
        rows = []
        for b in (8, 4, 2):
            cfg = base.replace(batch=b, name=f"{base.name}_b{b}")
            ds = DeviceStage(cfg, si.make_stage_inputs(cfg, seed=0))
            ds.step()
            blk = ds.stage.profile(ds.params, ds.x, ds.cc, ds.y, ds.dy, ds.dx, ds.d_cond, ds.dparams, ds.ws, reps=10)
            torch.cuda.synchronize()
            for rep in range(tiles):
                rows += [dict(r, layer=r["layer"] + rep * cfg.n_blocks) for r in blk]
            del ds
            torch.cuda.empty_cache()
        L = tiles * base.n_blocks
        prof = P.Profile(L, {}, {}, {}, {}, [0] * L, {})
        for r in rows:
            for name, tab in (("fwd_ms", prof.fwd_ms), ("bwd_ms", prof.bwd_ms), ("cf_bytes", prof.cf_bytes), ("cb_bytes", prof.cb_bytes)):
                tab.setdefault(r["batch"], [0] * L)[r["layer"]] = r[name]
            prof.grad_bytes[r["layer"]] = r["grad_bytes"]
            if r["layer"] == L - 1:
                prof.out_bytes[r["batch"]] = r["out_bytes"]
        profs.append(prof); all_rows.append(rows)
    link = dict(p2p_gbps=153.0, p2p_latency_ms=0.01, ar_gbps=7 * 153.0 / 2, ar_latency_ms=0.05)
    out = {"workload": "down: cfg2 blocks x3 (6 layers), up: cfg3 blocks x3 (6 layers), B=8, M_CDM=8, D=4", "links": link,
           "per_layer_ms": {n: {str(b): {"fwd": pr.fwd_ms[b][0], "bwd": pr.bwd_ms[b][0]} for b in sorted(pr.fwd_ms)} for n, pr in zip(("down", "up"), profs)},
           "plans": []}
    for uni in (False, True):
        t0 = time.perf_counter()
        for _ in range(5):
            got = binding.partition_solve_bidirectional(all_rows[0], all_rows[1], 8, 8, 4, uniform_replication=uni, **link)
        t_lib = (time.perf_counter() - t0) / 5
        o = P.Options(micro_batch=8, n_micro_batches=8, n_devices=4, uniform_replication=uni, **link)
        t0 = time.perf_counter()
        ref = P.solve_bidirectional(profs[0], profs[1], o)
        t_or = time.perf_counter() - t0
        same = (got["first_layer_down"], got["first_layer_up"], got["replicas"]) == (ref.first_layer_down, ref.first_layer_up, ref.replicas) \
            and abs(got["t_max_ms"] - ref.t_max_ms) <= 1e-9 * ref.t_max_ms
        out["plans"].append({"uniform_replication": uni, "layers_down": got["n_layers_down"], "layers_up": got["n_layers_up"], "replicas": got["replicas"],
                             "t0_ms": got["t0_ms"], "gap_ms": got["gap_ms"], "t_max_ms": got["t_max_ms"], "solve_ms_library": t_lib * 1e3,
                             "solve_ms_oracle": t_or * 1e3, "matches_oracle": same})
    return out


def bubble_report(si, DeviceStage, DeviceEncoder):
    """Bubble filling (Sec. 5) on measured profiles: the partition of --partition (self-conditioning off), one 1F1B
    iteration simulated from the measured stage times, and the frozen text encoder (profiled here at local batch 4..64,
    training batch = M x B = 256) placed into its bubbles.  The paper's 10 ms floor for a bubble assumes stages of
    hundreds of ms; these stages take 8 ms per micro-batch, so the floor is scaled to 0.1 ms."""
    import torch
    from paper_2405_01248_amd import binding
    from oracle import bubbles as Bu
    part, prof, _ = partition_report(si, DeviceStage)
    plan = part["plans"][0]
    S, reps, M, Bm = len(plan["replicas"]), plan["replicas"], 8, 32
    f, bw, cf = [], [], []
    lo = 0
    for s in range(S):
        b = Bm // reps[s]
        hi = lo + plan["layers_per_stage"][s]
        f.append(sum(prof.fwd_ms[b][lo:hi])); bw.append(sum(prof.bwd_ms[b][lo:hi]))
        if s:
            cf.append(prof.cf_bytes[b][lo - 1] / (part["links"]["p2p_gbps"] * 1e9) * 1e3 + part["links"]["p2p_latency_ms"])
        lo = hi
    cfg = si.CONFIG5
    de = DeviceEncoder(cfg, si.make_encoder_inputs(cfg, seed=0))
    batches = [4, 8, 12, 16, 24, 32, 48, 64]
    rows = de.enc.profile(de.params, de.ids, de.hidden, de.gb, batches, de.ws, reps=5)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    bubbles, t_iter = binding.bubbles_1f1b(f, bw, reps, M, cf or None, cf or None, None, 0.1)
    fills, summ = binding.bubbles_fill(bubbles, rows, M * Bm, sum(reps))
    t_lib = time.perf_counter() - t0
    nl = cfg.n_layers + 2
    comp = Bu.Component(nl, {b: [r["fwd_ms"] for r in rows if r["batch"] == b] for b in batches})
    t0 = time.perf_counter()
    busy, t = Bu.simulate_1f1b(f, bw, M, cf or None, cf or None)
    ref_b = Bu.find_bubbles(busy, t, reps, 0.1)
    ref = Bu.fill_all(ref_b, [comp], M * Bm, sum(reps))
    t_or = time.perf_counter() - t0
    same = len(bubbles) == len(ref_b) and abs(summ["filled_device_ms"] - ref.filled_device_ms) <= 1e-9 * max(ref.filled_device_ms, 1e-9) \
        and abs(summ["leftover_ms"] - ref.leftover_ms) <= 1e-9 * max(ref.leftover_ms, 1e-9)
    D = sum(reps)
    return {"workload": part["workload"], "stages": {"layers": plan["layers_per_stage"], "replicas": reps, "fwd_ms": f, "bwd_ms": bw, "comm_ms": cf},
            "iteration_ms": t_iter, "n_bubbles": len(bubbles), "bubble_ratio": summ["bubble_device_ms"] / (D * t_iter),
            "bubble_ratio_after_filling": (summ["bubble_device_ms"] - summ["filled_device_ms"]) / (D * (t_iter + summ["leftover_ms"])),
            "encoder_ms_at_local_batch": {str(b): sum(comp.fwd_ms[b]) for b in batches},
            "filled_device_ms": summ["filled_device_ms"], "bubble_device_ms": summ["bubble_device_ms"], "leftover_ms": summ["leftover_ms"],
            "placements": [(r["bubble"], r["first_layer"], r["n_layers"], r["samples"], r["partial"]) for r in fills],
            "solve_ms_library": t_lib * 1e3, "solve_ms_oracle": t_or * 1e3, "matches_oracle": same}


def search_report(si, DeviceStage, DeviceEncoder):
    """The search over stages, micro-batches and group size (Sec. 3, steps 2-5) on profiles measured here: the DiT backbone of
    --partition (28 layers, profiled at local batch 32 / 16 / 8 / 4) with self-conditioning at p = 0.5 and the frozen text
    encoder as the non-trainable part; 8 devices, training batch 256; group sizes 2 / 4 / 8, micro-batch counts 2 / 4 / 8 / 16."""
    import torch
    from paper_2405_01248_amd import binding
    from oracle import bubbles as Bu, search as S
    part, prof, rows = partition_report(si, DeviceStage)
    cfg = si.CONFIG5
    de = DeviceEncoder(cfg, si.make_encoder_inputs(cfg, seed=0))
    batches = [4, 8, 12, 16, 24, 32, 48, 64]
    enc_rows = de.enc.profile(de.params, de.ids, de.hidden, de.gb, batches, de.ws, reps=5)
    torch.cuda.synchronize()
    link = part["links"]
    kw = dict(world_size=8, training_batch=256, group_sizes=(2, 4, 8), micro_batch_counts=(2, 4, 8, 16), self_cond_prob=0.5,
              uniform_replication=True, min_bubble_ms=0.1, **link)
    t0 = time.perf_counter()
    cands, best = binding.schedule_search(rows + enc_rows, **kw)
    t_lib = time.perf_counter() - t0
    comp = Bu.Component(cfg.n_layers + 2, {b: [r["fwd_ms"] for r in enc_rows if r["batch"] == b] for b in batches})
    t0 = time.perf_counter()
    ref, ref_best = S.search(prof, [comp], S.SearchOptions(**kw))
    t_or = time.perf_counter() - t0
    same = len(cands) == len(ref) and best == ref_best and all(
        (c["n_stages"], c["n_micro_batches"], c["group_size"]) == (r.n_stages, r.n_micro_batches, r.group_size)
        and abs(c["iteration_ms"] - r.iteration_ms) <= 1e-9 * r.iteration_ms for c, r in zip(cands, ref))
    pick = lambda c: {k: c[k] for k in ("n_stages", "n_micro_batches", "group_size", "micro_batch", "n_layers", "replicas", "pipeline_ms", "leftover_ms",
                                        "iteration_ms", "bubble_ratio", "bubble_ratio_filled")}
    # iteration time is per pipeline group; a group of D devices trains 256 D / 8 samples per iteration
    rate = lambda c: 256.0 * c["group_size"] / 8 / c["iteration_ms"] * 1e3 * (8 / c["group_size"])
    ranked = sorted(range(len(cands)), key=lambda i: cands[i]["iteration_ms"])
    return {"workload": part["workload"] + ", world 8, training batch 256, p = 0.5", "n_candidates": len(cands), "best": pick(cands[best]),
            "best_samples_per_s_all_groups": rate(cands[best]), "runners_up": [pick(cands[i]) for i in ranked[1:4]],
            "solve_ms_library": t_lib * 1e3, "solve_ms_oracle": t_or * 1e3, "matches_oracle": same}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2", choices=["cfg2", "cfg3", "cfg4", "cfg5", "cfg6"])
    ap.add_argument("--slices", default=None,
                    help="encoder workloads (cfg5, cfg6): comma-separated slice sizes to time instead of all of the configuration's "
                         "(the full global batch is always included); keeps counter-collection runs short")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the short runs of the other workloads")
    ap.add_argument("--serial", action="store_true",
                    help="issue the backward's weight-gradient kernels in program order instead of on the side stream "
                         "(per-kernel profiling; the default overlaps them)")
    ap.add_argument("--fusion", type=int, default=None, choices=[0, 1, 2, 3],
                    help="GeGLU epilogue-fusion mask of the stage (library default when omitted); for A/B timing")
    ap.add_argument("--bubbles", action="store_true",
                    help="instead of the step benchmark: --partition's plan for cfg4, its 1F1B bubbles, and their filling with "
                         "the text encoder profiled here at the regular partial-batch sizes (library and oracle)")
    ap.add_argument("--fp8", action="store_true",
                    help="instead of the step benchmark: the FP8 (E4M3) projection GEMM beside the bf16 one on the workloads' projection shapes")
    ap.add_argument("--search", action="store_true",
                    help="instead of the step benchmark: the search over stages, micro-batches and group size (Sec. 3) on profiles measured on this GPU")
    ap.add_argument("--bidirectional", action="store_true",
                    help="instead of the step benchmark: the bidirectional partitioner (Sec. 4.2) on profiles of two backbones at different resolutions measured on this GPU")
    ap.add_argument("--partition", action="store_true",
                    help="instead of the step benchmark: profile the DiT stage's blocks at local batch sizes 32, 16, 8, 4 on this "
                         "GPU, tile them to a 28-layer backbone and run the partitioner (library and oracle) for 8 devices")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives are part of it); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import synth_inputs as si
    from paper_2405_01248_amd import load_library
    from paper_2405_01248_amd.harness import DeviceEncoder, DeviceStage
    load_library()        # fails loudly if the HIP library is missing
    torch.cuda.set_device(0)

    names = {"cfg2": si.CONFIG2, "cfg3": si.CONFIG3, "cfg4": si.CONFIG4}

    def run_stage(cfg, steps, warmup):
        ds = DeviceStage(cfg, si.make_stage_inputs(cfg, seed=0))
        if args.serial:
            ds.stage.set_overlap(False)
        if args.fusion is not None:
            ds.stage.set_fusion(args.fusion)
        med = {}
        sec = timed(ds.step, steps, warmup, med)
        fl = stage_flops(cfg)
        return ds, {"samples_per_s": cfg.batch / sec, "ms_per_step": sec * 1e3, "median_ms_per_step": med["ms"], "tflops": fl / sec / 1e12,
                    "mfma_peak_frac": fl / sec / MFMA_PEAK}

    def slice_list(c):
        if not args.slices:
            return c.slices
        want = sorted({int(v) for v in args.slices.split(",")} | {c.global_batch})
        bad = [b for b in want if b <= 0 or c.global_batch % b]
        if bad:
            raise SystemExit(f"--slices: {bad} do not divide the global batch {c.global_batch}")
        return tuple(want)

    def run_encoder(steps, warmup):
        c = si.CONFIG5
        de = DeviceEncoder(c, si.make_encoder_inputs(c, seed=0))
        out = {}
        for b in slice_list(c):
            sec = timed(lambda: de.run_slices(b), steps, warmup)
            out[str(b)] = {"samples_per_s": c.global_batch / sec, "ms_per_global_batch": sec * 1e3,
                           "ms_per_call": sec * 1e3 * b / c.global_batch,
                           "mfma_peak_frac": encoder_flops_per_sample(c) * c.global_batch / sec / MFMA_PEAK}
        return de, out

    def run_image_encoder(steps, warmup):
        from paper_2405_01248_amd.harness import DeviceImageEncoder
        c = si.CONFIG6
        de = DeviceImageEncoder(c, si.make_image_encoder_inputs(c, seed=0, weight_std=0.0))
        out = {}
        for b in slice_list(c):
            sec = timed(lambda: de.run_slices(b), steps, warmup)
            out[str(b)] = {"samples_per_s": c.global_batch / sec, "ms_per_global_batch": sec * 1e3,
                           "ms_per_call": sec * 1e3 * b / c.global_batch,
                           "mfma_peak_frac": image_encoder_flops_per_sample(c) * c.global_batch / sec / MFMA_PEAK}
        return de, out

    if args.fp8:
        print(json.dumps(fp8_report()))
        return
    if args.search:
        print(json.dumps(search_report(si, DeviceStage, DeviceEncoder)))
        return
    if args.bidirectional:
        print(json.dumps(bidirectional_report(si, DeviceStage)))
        return
    if args.partition:
        print(json.dumps(partition_report(si, DeviceStage)[0]))
        return
    if args.bubbles:
        print(json.dumps(bubble_report(si, DeviceStage, DeviceEncoder)))
        return

    result = {"n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": True, "scaling": "weak",
              "vs_baseline": None, "dtype": "bf16", "data": "synthetic"}
    if args.workload == "cfg6":
        de, enc = run_image_encoder(max(2, args.steps // 3), max(1, args.warmup // 2))
        full = enc[str(si.CONFIG6.global_batch)]
        result.update(metric="image_encoder_fwd_samples_per_sec", value=full["samples_per_s"], unit="samples/s",
                      ms_per_step=full["ms_per_global_batch"], mfma_peak_frac=full["mfma_peak_frac"],
                      config={"workload": si.CONFIG6.name, "global_batch": si.CONFIG6.global_batch, "slice_sizes": enc,
                              "algorithmic_tflop_per_sample": image_encoder_flops_per_sample(si.CONFIG6) / 1e12})
        del de
    elif args.workload == "cfg5":
        de, enc = run_encoder(args.steps, args.warmup)
        full = enc[str(si.CONFIG5.global_batch)]
        result.update(metric="encoder_fwd_samples_per_sec", value=full["samples_per_s"], unit="samples/s",
                      ms_per_step=full["ms_per_global_batch"],
                      config={"workload": si.CONFIG5.name, "global_batch": 64, "slice_sizes": enc})
        del de
    else:
        cfg = names[args.workload]
        ds, r = run_stage(cfg, args.steps, args.warmup)
        result.update(metric="stage_fwd_bwd_samples_per_sec", value=r["samples_per_s"], unit="samples/s",
                      ms_per_step=r["ms_per_step"], median_ms_per_step=r["median_ms_per_step"], mfma_peak_frac=r["mfma_peak_frac"],
                      achieved_tflops=r["tflops"],
                      config={"workload": cfg.name, "micro_batch": cfg.batch, "tokens": cfg.tokens, "d_model": cfg.d_model,
                              "n_blocks": cfg.n_blocks, "self_conditioning": cfg.self_cond,
                              "algorithmic_tflop_per_step": stage_flops(cfg) / 1e12})
        del ds
    torch.cuda.empty_cache()

    if not args.no_others:
        others = {}
        for k, c in names.items():
            if k != args.workload:
                ds, r = run_stage(c, max(3, args.steps // 3), 2)
                others[c.name] = r
                del ds
                torch.cuda.empty_cache()
        if args.workload != "cfg5":
            de, enc = run_encoder(max(3, args.steps // 3), 2)
            others[si.CONFIG5.name] = enc
            del de
        result["other_workloads"] = others

    # Roofline of the dominant kernel: a separate instrumented pass of the same workload in the
    # same launch configuration, with HIP events around every launch on the launch stream.
    result["roofline"], result["kernel_classes"] = kernel_roofline(args.workload, names, si, DeviceStage, DeviceEncoder)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline_image_encoder(si.CONFIG6) if args.workload == "cfg6" else cpu_baseline_stage(names.get(args.workload, si.CONFIG2))
    print(json.dumps(result))


if __name__ == "__main__":
    main()

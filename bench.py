#!/usr/bin/env python3
"""Benchmark of the MoE-offloading decode step on one MI355X.

A "step" is one decode token (batch B) through the whole hot path of every layer of the workload:
RMSNorm + gate + top-2, LRU cache resolve, demand copies of missed experts from pinned host memory,
speculative prefetch for the next layer, fused dequant-GEMV expert FFN, combine + residual.

Prints ONE JSON line: metric = decode tokens/s of the whole job, plus
  roofline      -- the fused dequant-GEMV as a whole (w1,w3 -> SiLU*mul -> w2 -> combine: both of its kernels, the
                   bytes of both over the sum of their durations) against MI355X's 8 TB/s HBM peak; algorithmic bytes
                   per launch / average launch duration (HIP events on the compute stream); roofline_w13 and
                   roofline_w2 give the two kernels one by one;
  ablations     -- the same workload, fewer steps, with whole-expert speculative loads (the paper's literal
                   algorithm; the headline run moves a 4 MiB head first) and without speculative loading;
  cpu_baseline  -- the CPU oracle timed on the host cores on a bounded sample of the same workload.
All inputs are synthetic and seeded (see workload/); hidden states are resident in HBM before timing.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
# HBM bytes per launch (read + written) of the dominant kernel from hardware counters, valid for the default
# workload and launch shape only (4-bit g64 Mixtral experts, batch 1): FETCH_SIZE and WRITE_SIZE of two
# rocprofv3 --pmc runs, scaled by the copy probe; see profiles/hbm_traffic_gemv_kernels_4bit.md
PMC_TRAFFIC_W13_4BIT_B1 = 132_465_708
PMC_TRAFFIC_W2_4BIT_B1 = 67_301_016     # k_w2_token: 67,276,440 B read + 24,576 B written
PMC_TRAFFIC_FFN_4BIT_B1 = None   # the one-launch kernels are not the default; their counters were not collected
LINK_PEAK_GBS = 64.0           # PCIe Gen5 x16, one direction, nominal


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def build_model(shape, formats, batch, device, keep_layers, n_staging=4, swap=False, scale_group=0):
    import torch
    import workload as W
    from paper_2312_17238_amd.engine import Stack, layer_config

    gates = [W.gate_weight(shape.seed, l, shape.n_experts, shape.hidden) for l in range(shape.layers)]
    gamma = [W.rms_gamma(shape.hidden) for _ in range(shape.layers)] if shape.rms_eps > 0 else None
    from paper_2312_17238_amd import binding as B
    cfgs = [layer_config(shape.hidden, shape.ffn, shape.n_experts, shape.top_k, formats[l][0], formats[l][1],
                         shape.cache_slots, shape.prefetch_m, shape.rms_eps, 1 if swap else 0,
                         B.MOE_LAYER_SWAP if swap else 0, scale_group) for l in range(shape.layers)]
    stack = Stack(cfgs, gates, gamma, n_staging=n_staging, max_batch=batch, device=device)
    kept = {}
    t0 = time.time()
    for l in range(shape.layers):
        bits, group = formats[l]
        for e in range(shape.n_experts):
            mats = W.quantized_expert(shape.seed, l, e, shape.hidden, shape.ffn, bits, group, device, scale_group)
            for m, mat in enumerate(mats):
                stack.load_expert(l, e, m, *mat)
            if l in keep_layers:
                kept[(l, e)] = [tuple(t.cpu().numpy() if hasattr(t, "cpu") else t for t in mat) for mat in mats]
            del mats
        if l % 4 == 3 or l + 1 == shape.layers:
            log(f"generated, quantized and loaded layers 0..{l} ({time.time() - t0:.1f} s)")
    return stack, gates, gamma, kept


def cpu_baseline(shape, formats, gates, gamma, kept, xs, budget_s=20.0):
    """Time the CPU oracle (numpy gate + plain-C fp64 FFN, OpenMP over rows) on (token, layer) steps of
    the first kept layers, free-running from the same inputs; report tokens/s scaled to the full stack."""
    import numpy as np
    from oracle import c_ffn
    from oracle import moe_oracle as O

    layers = sorted({l for l, _ in kept})
    done, t0 = 0, time.time()
    tokens = 0
    for t in range(xs.shape[0]):
        for b in range(xs.shape[1]):
            x = xs[t, b].numpy()
            for l in layers:
                experts = {e: kept[(l, e)] for e in range(shape.n_experts)}
                r = O.moe_block(x, gates[l].numpy(), experts, formats[l][1], shape.top_k,
                                gamma[l].numpy() if gamma else None, shape.rms_eps, ffn=c_ffn.expert_ffn)
                x = r.x_out
                done += 1
            tokens += 1
        if time.time() - t0 > budget_s:
            break
    dt = time.time() - t0
    steps_per_token = shape.layers
    return {"value": (done / steps_per_token) / dt, "unit": "tokens/s", "cores": c_ffn.threads(), "kind": "oracle",
            "sample": f"{done} (token, layer) steps on layers {layers[0]}..{layers[-1]} ({tokens} tokens), "
                      f"{dt:.1f} s, scaled by {steps_per_token} layers per token"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=512)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default="mixtral_stack",
                    choices=["tiny", "mixtral_layer", "mixtral_stack", "mixtral_stack_lowbit", "mixtral_stack_batched"])
    ap.add_argument("--batch", type=int, default=0, help="tokens per step (default: the workload's)")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers (debugging only)")
    ap.add_argument("--cache-slots", type=int, default=0)
    ap.add_argument("--prefetch", type=int, default=-1, help="m: experts guessed per layer (0 = ablation without pre-loading)")
    ap.add_argument("--no-cache", action="store_true", help="ablation without LRU cache (and usually --prefetch 0)")
    ap.add_argument("--bits", type=int, default=0, help="override the expert format: 4, 3 or 2 bits (with --group)")
    ap.add_argument("--group", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true", help="do not record HIP events around the engine's launches")
    ap.add_argument("--copy-event-stride", type=int, default=7,
                    help="time only every n-th expert transfer with HIP events (1: all; the event pairs slow a saturated link by ~1 %%)")
    ap.add_argument("--spec-head-mb", type=int, default=4,
                    help="speculative loads copy only the first N MiB until the guess is confirmed (0: whole expert, as in the paper)")
    ap.add_argument("--mfma-form", type=int, default=0, help="matrix-core kernel form 1..5 (0: the library's default)")
    ap.add_argument("--mfma16-waves", type=int, default=0, help="waves per block of the 16-token matrix-core kernels, 4 or 8 (0: the library's default)")
    ap.add_argument("--mfma-min-batch", type=int, default=0, help="batches at least this large run on the matrix cores (0: the library's default)")
    ap.add_argument("--fused", type=int, default=-1,
                    help="single-token steps run w1/w3 and w2 as one persistent launch: 1 with a grid barrier, 2 expert after expert; 0 two launches (-1: the library's default)")
    ap.add_argument("--no-token-path", action="store_true", help="single-token steps use the general kernels (atomics + residual kernel)")
    ap.add_argument("--no-probe", action="store_true", help="skip the plain streaming-read / copy calibration kernels")
    ap.add_argument("--ablation-steps", type=int, default=64,
                    help="steps of each ablation run after the timed one (whole-expert speculative loads; no speculative loading); 0: none")
    ap.add_argument("--scale-group", type=int, default=0,
                    help="two-level metadata (Sec. 4.2): 8-bit scale and zero codes with an fp16 quad per run of this many "
                         "groups (256 for the paper's 4-bit scheme); 4-bit formats only, 4.25 instead of 4.5 bits per weight")
    ap.add_argument("--swap", action="store_true",
                    help="hosts that cannot hold every expert (Sec. 3.3): experts split between host and device buffers, "
                         "every load writes the evicted expert back (experts 0..k-1 start on the device)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (one process, no collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        return 2

    import dataclasses
    import numpy as np
    import torch
    import workload as W
    from paper_2312_17238_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    shape = W.CONFIGS[args.workload]
    if args.layers:
        shape = dataclasses.replace(shape, layers=args.layers)
    if args.cache_slots:
        shape = dataclasses.replace(shape, cache_slots=args.cache_slots)
    if args.prefetch >= 0:
        shape = dataclasses.replace(shape, prefetch_m=args.prefetch)
    batch = args.batch or (1 if args.workload != "mixtral_stack_batched" else shape.batch)
    if args.bits:
        shape = dataclasses.replace(shape, bits=args.bits, group=args.group or {4: 64, 3: 64, 2: 16}[args.bits])
    formats = W.layer_formats(shape)
    device = "cuda:0"
    n_tok = args.warmup + args.steps
    keep_layers = set() if args.no_cpu_baseline else set(range(min(2, shape.layers)))
    log(f"workload {shape.name}: {shape.layers} layers, H={shape.hidden}, F={shape.ffn}, E={shape.n_experts}, "
        f"k={shape.cache_slots}, m={shape.prefetch_m}, batch={batch}, formats={sorted(set(formats))}")
    stack, gates, gamma, kept = build_model(shape, formats, batch, device, keep_layers, swap=args.swap,
                                            scale_group=args.scale_group)
    if args.no_cache:
        stack.set_flags(B.MOE_LAYER_NO_CACHE)
    B.moe_ctx_set_option(stack.ctx, "spec_head_mb", args.spec_head_mb)
    if args.mfma_form:
        B.moe_ctx_set_option(stack.ctx, "mfma_form", args.mfma_form)
    if args.mfma16_waves:
        B.moe_ctx_set_option(stack.ctx, "mfma16_waves", args.mfma16_waves)
    if args.mfma_min_batch:
        B.moe_ctx_set_option(stack.ctx, "mfma_min_batch", args.mfma_min_batch)
    if args.fused >= 0:
        B.moe_ctx_set_option(stack.ctx, "fused", args.fused)
    if args.no_token_path:
        B.moe_ctx_set_option(stack.ctx, "token_path", 0)
    xs = (W.hidden_iid if shape.hidden_kind == "iid" else W.hidden_ar1)(shape.seed, n_tok, batch, shape.hidden)
    x_dev = xs.to(device)                                   # inputs resident in HBM before the timed region
    x_out = torch.empty(batch, shape.hidden, dtype=torch.float16, device=device)
    torch.cuda.synchronize()

    probe = None
    if not args.no_probe:
        # calibration: a plain streaming read (the practical HBM ceiling on this machine) and a plain copy of
        # known size (the kernel hardware-counter readings are scaled by)
        src = torch.empty(4 << 30, dtype=torch.uint8, device=device).zero_()
        dst = torch.empty(1 << 30, dtype=torch.uint8, device=device)
        s0 = torch.cuda.current_stream().cuda_stream
        ms_r = B.moe_probe_bandwidth(src.data_ptr(), None, 4 << 30, 16384, 5, s0)
        ms_c = B.moe_probe_bandwidth(src.data_ptr(), dst.data_ptr(), 1 << 30, 8192, 3, s0)
        probe = {"read_gbs": (4 << 30) / ms_r / 1e6, "read_bytes": 4 << 30,
                 "copy_gbs_each_way": (1 << 30) / ms_c / 1e6, "copy_bytes": 1 << 30}
        # what a launch of the size of the two GEMV kernels can reach at all: the same plain read over exactly the
        # algorithmic bytes of one launch of each (w1/w3 and w2 of top_k experts at batch 1), one launch at a time,
        # each over another part of the 4 GiB buffer so that nothing comes from the memory-side cache; median of 9,
        # best of three grid sizes.  A launch this short never reaches the steady-state rate above.
        if batch == 1:
            l0 = stack.cfgs[0]
            # bytes of w2 and of w1+w3 of one expert, from the blob size: rows of w2 are ffn codes + metadata, of w1/w3 hidden codes + metadata
            per_w = {4: 0.5, 3: 0.375, 2: 0.25}[l0.bits]
            meta = (2 if l0.scale_group else 4) / l0.group
            w2_bytes = int(shape.top_k * l0.hidden * l0.ffn * (per_w + meta)) // 256 * 256
            w13_bytes = 2 * w2_bytes
            def same_size(nbytes):
                best = None
                for blocks in (512, 2048, 4096):
                    ts = sorted(B.moe_probe_bandwidth(src.data_ptr() + ((i * 409_600_000) % ((4 << 30) - nbytes)) // 256 * 256, None, nbytes, blocks, 1, s0)
                                for i in range(9))
                    best = ts[4] if best is None else min(best, ts[4])
                return 1e3 * best
            probe["read_us_at_w13_launch_bytes"] = same_size(w13_bytes)
            probe["read_us_at_w2_launch_bytes"] = same_size(w2_bytes)
            probe["w13_launch_bytes"], probe["w2_launch_bytes"] = w13_bytes, w2_bytes
        del src, dst
        torch.cuda.empty_cache()
        # the host link alone: pinned -> device copies of one expert blob, back to back on one stream
        blob = max(stack.blob_bytes)
        hsrc = torch.empty(blob, dtype=torch.uint8, pin_memory=True).zero_()
        ddst = torch.empty(blob, dtype=torch.uint8, device=device)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ddst.copy_(hsrc, non_blocking=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(8):
            ddst.copy_(hsrc, non_blocking=True)
        e1.record()
        torch.cuda.synchronize()
        probe["h2d_gbs"] = 8 * blob / e0.elapsed_time(e1) / 1e6
        probe["h2d_bytes_per_copy"] = blob
        del hsrc, ddst
        torch.cuda.empty_cache()
        log(f"probe: streaming read {probe['read_gbs']:.0f} GB/s, copy {probe['copy_gbs_each_way']:.0f} GB/s each way, "
            f"pinned host->device {probe['h2d_gbs']:.1f} GB/s")

    for t in range(args.warmup):
        stack.step(x_dev[t], x_out)
    stack.synchronize()
    torch.cuda.synchronize()
    before = stack.total_stats()
    layers_before = stack.stats()
    if not args.no_profile:
        B.moe_ctx_set_option(stack.ctx, "profile_copy_stride", max(1, args.copy_event_stride))
        B.moe_ctx_profile_enable(stack.ctx, True)
    t0 = time.perf_counter()
    for t in range(args.warmup, n_tok):
        stack.step(x_dev[t], x_out)
    stack.synchronize()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    after = stack.total_stats()
    layers_after = stack.stats()
    prof = None if args.no_profile else B.moe_ctx_profile_read(stack.ctx).as_dict()
    if not args.no_profile:
        B.moe_ctx_profile_enable(stack.ctx, False)
    d = {k: after[k] - before[k] for k in after}
    assert np.isfinite(x_out.float().cpu().numpy()).all()

    tokens = args.steps * batch
    result = {
        "metric": "MoE decode tokens/s (32-layer Mixtral-shape, 4-bit, LRU k=2); GEMV HBM GB/s",
        "value": tokens / dt, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * dt / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{shape.name}: {shape.layers} layers, hidden {shape.hidden}, ffn {shape.ffn}, "
                               f"{shape.n_experts} experts top-{shape.top_k}, formats {sorted(set(formats))}, "
                               f"LRU k={shape.cache_slots}, prefetch m={shape.prefetch_m}, b=4 staging buffers, "
                               f"batch {batch}, {shape.hidden_kind} hidden states, seed {shape.seed}",
                   "no_cache": bool(args.no_cache), "spec_head_mb": args.spec_head_mb, "swap": bool(args.swap),
                   "scale_group": args.scale_group, "expert_blob_bytes": max(stack.blob_bytes)},
    }
    link_bytes = d["bytes_h2d_demand"] + d["bytes_h2d_spec"]
    per_layer = [{k: a[k] - b[k] for k in ("needed", "hits", "prefetch_hits")} for a, b in zip(layers_after, layers_before)]
    # Sec. 4.1's recall counts an expert as "already available on GPU".  With head-then-tail speculative loads a
    # confirmed guess has only its head there (requested, in flight or landed) when the gate decides; the rest
    # crosses the link after the decision.  resident_byte_frac weighs every needed expert by the bytes that were
    # on the device (or on their way) at decision time.
    head = args.spec_head_mb << 20
    on_dev = sum(x["hits"] * bb + x["prefetch_hits"] * (min(head, bb) if head else bb) for x, bb in zip(per_layer, stack.blob_bytes))
    all_needed = sum(x["needed"] * bb for x, bb in zip(per_layer, stack.blob_bytes))
    result["cache"] = {"needed": d["needed"], "hits": d["hits"], "prefetch_hits": d["prefetch_hits"], "misses": d["misses"],
                       "prefetch_hits_fully_staged": 0 if head else d["prefetch_hits"],
                       "prefetch_hits_head_only": d["prefetch_hits"] if head else 0,
                       "spec_issued": d["spec_issued"], "spec_wasted": d["spec_wasted"],
                       "recall": (d["hits"] + d["prefetch_hits"]) / max(1, d["needed"]),
                       "lru_hit_ratio": d["hits"] / max(1, d["needed"]),
                       "resident_byte_frac": on_dev / max(1, all_needed),
                       "link_bytes_per_token": link_bytes / tokens}
    # per layer: LRU hit ratio and recall (hits + prefetch hits) over the timed steps
    result["cache"]["per_layer_hit_ratio"] = [round(x["hits"] / max(1, x["needed"]), 3) for x in per_layer]
    result["cache"]["per_layer_recall"] = [round((x["hits"] + x["prefetch_hits"]) / max(1, x["needed"]), 3) for x in per_layer]
    # the step can be no faster than its bytes over the slower of the two pipes (nominal peaks)
    hbm_bytes_per_token = 2.0 * sum(stack.blob_bytes) * batch / max(1, batch) if batch == 1 else None
    t_link = (link_bytes / tokens) / (LINK_PEAK_GBS * 1e9)
    t_hbm = (hbm_bytes_per_token / (HBM_PEAK_GBS * 1e9)) if hbm_bytes_per_token else 0.0
    bound_tps = 1.0 / max(t_link, t_hbm, 1e-12)
    result["step_bound"] = {"tokens_per_s_at_nominal_peaks": bound_tps, "frac": (tokens / dt) / bound_tps,
                            "link_s_per_token": t_link, "hbm_s_per_token": t_hbm if hbm_bytes_per_token else None}
    if prof and prof["ffn"]["launches"]:
        # single-token steps run the expert FFN as one persistent launch: that kernel is the dominant one
        ff, cp, gt = prof["ffn"], prof["copy"], prof["gate"]
        ach = ff["bytes"] / max(ff["total_ms"], 1e-9) / 1e6
        result["roofline"] = {"bound": "hbm", "kernel": "k_ffn_seq (w1,w3 -> SiLU*mul -> w2 -> combine -> residual in one launch, expert after expert)" if args.fused == 2
                              else "k_ffn_token (w1,w3 -> SiLU*mul -> grid barrier -> w2 -> combine -> residual)",
                              "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                              "traffic": PMC_TRAFFIC_FFN_4BIT_B1 if (batch == 1 and set(formats) == {(4, 64)}
                                                                     and shape.hidden == 4096 and shape.ffn == 14336) else None,
                              "launches": ff["launches"], "bytes_per_launch": ff["bytes"] / ff["launches"],
                              "avg_us": 1e3 * ff["total_ms"] / ff["launches"],
                              "measured_read_probe_gbs": probe["read_gbs"] if probe else None}
        result["gemv_hbm_gbs"] = ach
    elif prof:
        w13, w2 = prof["w13"], prof["w2"]
        matrix_cores = batch >= 16 and set(formats) == {(4, 64)}
        default_shape = (batch == 1 and set(formats) == {(4, 64)} and not args.scale_group and shape.hidden == 4096
                         and shape.ffn == 14336 and not args.no_token_path)

        def kernel_line(pr, name, traffic):
            ach = pr["bytes"] / max(pr["total_ms"], 1e-9) / 1e6      # GB/s
            return {"bound": "hbm", "kernel": name, "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                    "traffic": traffic if default_shape else None, "launches": pr["launches"],
                    "bytes_per_launch": pr["bytes"] / max(1, pr["launches"]), "avg_us": 1e3 * pr["total_ms"] / max(1, pr["launches"])}

        n13 = "k_mfma_stream_q4<W13> (grouped dequant-GEMM w1,w3 -> SiLU*mul)" if matrix_cores else "k_w13 (fused dequant-GEMV w1,w3 -> SiLU*mul)"
        n2 = ("k_mfma_stream_q4<W2> (grouped dequant-GEMM w2; k_combine adds and applies the residual)" if matrix_cores
              else "k_w2_token / k_w2 (fused dequant-GEMV w2 -> combine -> residual)")
        result["roofline_w13"] = kernel_line(w13, n13, PMC_TRAFFIC_W13_4BIT_B1)
        result["roofline_w2"] = kernel_line(w2, n2, PMC_TRAFFIC_W2_4BIT_B1)
        # the fused dequant-GEMV as the metric names it: both kernels, bytes of both over the sum of their durations,
        # per layer-step (one launch of each)
        both = (w13["bytes"] + w2["bytes"]) / max(w13["total_ms"] + w2["total_ms"], 1e-9) / 1e6
        steps_l = max(1, min(w13["launches"], w2["launches"]))
        result["roofline"] = {"bound": "hbm", "kernel": f"{n13} + {n2}", "achieved": both, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": both / HBM_PEAK_GBS,
                              "traffic": (PMC_TRAFFIC_W13_4BIT_B1 + PMC_TRAFFIC_W2_4BIT_B1) if default_shape else None,
                              "launches": steps_l, "bytes_per_launch": (w13["bytes"] + w2["bytes"]) / steps_l,
                              "avg_us": 1e3 * (w13["total_ms"] + w2["total_ms"]) / steps_l,
                              "measured_read_probe_gbs": probe["read_gbs"] if probe else None}
        if probe and "read_us_at_w13_launch_bytes" in probe and not matrix_cores:
            # the two launches against two plain reads of their sizes on this machine
            plain = probe["read_us_at_w13_launch_bytes"] + probe["read_us_at_w2_launch_bytes"]
            result["roofline"]["plain_read_us_at_launch_sizes"] = plain
            result["roofline"]["frac_of_plain_read_at_launch_sizes"] = plain / result["roofline"]["avg_us"]
        result["gemv_hbm_gbs"] = both
    if prof:
        cp, gt = prof["copy"], prof["gate"]
        if cp["launches"]:
            # rate over the transfers that were timed (every n-th); busy time = all bytes at that rate
            ac = cp["bytes"] / max(cp["total_ms"], 1e-9) / 1e6
            result["link"] = {"bound": "host-link", "achieved": ac, "peak": LINK_PEAK_GBS, "unit": "GB/s",
                              "frac": ac / LINK_PEAK_GBS, "copies_timed": cp["launches"],
                              "copy_event_stride": max(1, args.copy_event_stride),
                              "measured_h2d_probe_gbs": probe.get("h2d_gbs") if probe else None,
                              "busy_frac_of_wall": (link_bytes / (ac * 1e9)) / dt,
                              "wall_gbs": link_bytes / dt / 1e9}
        wb = prof["writeback"]
        if wb["launches"]:
            aw = wb["bytes"] / max(wb["total_ms"], 1e-9) / 1e6
            result["link_writeback"] = {"bound": "host-link (device to host)", "achieved": aw, "peak": LINK_PEAK_GBS, "unit": "GB/s",
                                        "frac": aw / LINK_PEAK_GBS, "copies_timed": wb["launches"],
                                        "busy_frac_of_wall": (d["bytes_d2h_writeback"] / (aw * 1e9)) / dt,
                                        "bytes_per_token": d["bytes_d2h_writeback"] / tokens}
        result["gate_avg_us"] = 1e3 * gt["total_ms"] / max(1, gt["launches"])
    if probe:
        result["probe"] = probe
    if args.ablation_steps > 0 and shape.prefetch_m > 0 and not args.swap and not args.no_cache:
        # Table 2's rows on the same inputs: the literal algorithm of Sec. 3.2/3.3 (a guessed expert is loaded whole)
        # and no speculative loading at all, each from a cold cache over the first tokens of the stream
        def short_run(head_mb, m):
            n = min(args.ablation_steps, n_tok - 8)
            stack.reset()
            B.moe_ctx_set_option(stack.ctx, "spec_head_mb", head_mb)
            stack.set_prefetch(m)
            for t in range(8):
                stack.step(x_dev[t], x_out)
            stack.synchronize()
            b0 = stack.total_stats()
            t1 = time.perf_counter()
            for t in range(8, 8 + n):
                stack.step(x_dev[t], x_out)
            stack.synchronize()
            torch.cuda.synchronize()
            el = time.perf_counter() - t1
            dd = {k: v - b0[k] for k, v in stack.total_stats().items()}
            return {"tokens_per_s": n * batch / el, "steps": n, "spec_head_mb": head_mb, "prefetch_m": m,
                    "recall": (dd["hits"] + dd["prefetch_hits"]) / max(1, dd["needed"]),
                    "link_bytes_per_token": (dd["bytes_h2d_demand"] + dd["bytes_h2d_spec"]) / (n * batch)}
        log("ablations: whole-expert speculative loads, no speculative loads, and the headline setting over the same steps")
        result["ablations"] = {"literal_whole_expert_speculation": short_run(0, shape.prefetch_m),
                               "without_speculative_loading": short_run(args.spec_head_mb, 0),
                               "as_timed_above": short_run(args.spec_head_mb, shape.prefetch_m)}
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a bounded sample")
        result["cpu_baseline"] = cpu_baseline(shape, formats, gates, gamma, kept, xs)
    stack.close()
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())

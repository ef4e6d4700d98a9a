"""When the expert transfers and the gate kernels of one decode step ran: a timeline from the engine's own events.

    python -m paper_2312_17238_amd.step_timeline [--workload mixtral_stack_batched] [--batch 1024] [--layers 6]
                                                 [--prefetch M] [--spec-head-mb N] [--warmup 3]

Builds the synthetic stack, runs a few warm-up steps, then one step with per-launch events switched on, and
prints every transfer and gate launch with its start (ms after the step began) and duration, marking where the host
link sat idle between two transfers; last the link's busy share of the step and the kernels' total.  It is how
the schedule of prompt-sized steps (resident experts first, guarded transfers, arriving experts one by one) was
found and checked.  Needs a GPU and the built library; imports nothing of the test infrastructure.
"""
from __future__ import annotations

import argparse
import dataclasses
import os
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workload as W  # noqa: E402
from paper_2312_17238_amd import binding as B  # noqa: E402
from paper_2312_17238_amd.engine import Stack, layer_config  # noqa: E402

KINDS = {0: "gate", 1: "w1/w3", 2: "w2", 3: "COPY", 5: "WRITE-BACK"}


def build(shape, formats, batch: int, device: str) -> Stack:
    gates = [W.gate_weight(shape.seed, l, shape.n_experts, shape.hidden) for l in range(shape.layers)]
    gamma = [W.rms_gamma(shape.hidden) for _ in range(shape.layers)] if shape.rms_eps > 0 else None
    cfgs = [layer_config(shape.hidden, shape.ffn, shape.n_experts, shape.top_k, formats[l][0], formats[l][1],
                         shape.cache_slots, shape.prefetch_m, shape.rms_eps) for l in range(shape.layers)]
    stack = Stack(cfgs, gates, gamma, n_staging=4, max_batch=batch, device=device)
    for l in range(shape.layers):
        for e in range(shape.n_experts):
            mats = W.quantized_expert(shape.seed, l, e, shape.hidden, shape.ffn, formats[l][0], formats[l][1], device)
            for m, mat in enumerate(mats):
                stack.load_expert(l, e, m, *mat)
            del mats
    return stack


def timeline(stack: Stack, x: torch.Tensor, x_out: torch.Tensor):
    """[(start ms, stop ms, kind)] of one step, sorted by start."""
    B.moe_ctx_set_option(stack.ctx, "profile_copy_stride", 1)
    B.moe_ctx_profile_enable(stack.ctx, True)
    stack.step(x, x_out)
    stack.synchronize()
    ev = [(a, b, name) for k, name in KINDS.items() for a, b in B.moe_ctx_profile_timeline(stack.ctx, k)]
    B.moe_ctx_profile_enable(stack.ctx, False)
    return sorted(ev)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="mixtral_stack_batched", choices=sorted(W.CONFIGS))
    ap.add_argument("--batch", type=int, default=1024)
    ap.add_argument("--layers", type=int, default=6)
    ap.add_argument("--prefetch", type=int, default=-1)
    ap.add_argument("--spec-head-mb", type=int, default=0)
    ap.add_argument("--warmup", type=int, default=3)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        print("step_timeline: no GPU visible", file=sys.stderr)
        return 2
    shape = dataclasses.replace(W.CONFIGS[args.workload], layers=args.layers)
    if args.prefetch >= 0:
        shape = dataclasses.replace(shape, prefetch_m=args.prefetch)
    stack = build(shape, W.layer_formats(shape), args.batch, "cuda:0")
    B.moe_ctx_set_option(stack.ctx, "spec_head_mb", args.spec_head_mb)
    xs = (W.hidden_iid if shape.hidden_kind == "iid" else W.hidden_ar1)(shape.seed, args.warmup + 1, args.batch, shape.hidden).to("cuda:0")
    x_out = torch.empty(args.batch, shape.hidden, dtype=torch.float16, device="cuda:0")
    for t in range(args.warmup):
        stack.step(xs[t], x_out)
    stack.synchronize()
    ev = timeline(stack, xs[args.warmup], x_out)
    print(f"{shape.name}: {shape.layers} layers, k={shape.cache_slots}, m={shape.prefetch_m}, batch {args.batch}, "
          f"speculative head {args.spec_head_mb} MiB; start ms, duration ms")
    last_end = None
    for a, b, name in ev:
        if name in ("w1/w3", "w2"):
            continue
        note = ""
        if name == "COPY":
            if last_end is not None and a - last_end > 0.05:
                note = f"   <-- link idle {a - last_end:.2f} ms"
            last_end = b
        print(f"{a:9.2f} {b - a:8.2f}  {name}{note}")
    copies = [(a, b) for a, b, n in ev if n == "COPY"]
    span = ev[-1][1] - ev[0][0]
    if copies:
        print(f"link busy {sum(b - a for a, b in copies):.2f} of {span:.2f} ms ({sum(b - a for a, b in copies) / span:.1%})")
    print(f"w1/w3 + w2 kernels {sum(b - a for a, b, n in ev if n in ('w1/w3', 'w2')):.2f} ms")
    stack.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())

"""Cache and speculative-loading recall on the synthetic stack: the analogue of the paper's Fig. 2.

    python -m paper_2312_17238_amd.recall_study [--workload mixtral_stack] [--tokens 128]

Runs the engine once over the workload with every expert resident (the outputs do not depend on the cache
size, Sec. 3.2), recording for every (token, layer) the routing decision and the gate input h.  From that record:

  * LRU hit ratio for k = top_k..E cached experts per layer (Sec. 3.1, Fig. 2 left): the recorded routing is
    replayed through the library's own cache bookkeeping in a context without a GPU;
  * recall of speculative loading (Sec. 3.2, Fig. 2 right): the gate of layer l+a applied to the gate input of
    layer l, a = 1, 2 and 10 layers ahead, guessing m = 1, 2 or 4 experts; recall = guessed and needed / needed.
    The guesses are the library's own: moe_layer_prefetch(layer l+a, h_l) runs the gate kernel and the top-m
    selection of the decode path and reports them most likely first, so the first m of four are the guess for m.

Prints one JSON object.  Needs a GPU and the built library; imports nothing of the test infrastructure.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workload as W  # noqa: E402
from paper_2312_17238_amd import binding as B  # noqa: E402
from paper_2312_17238_amd.engine import Stack, layer_config  # noqa: E402


def record(shape, formats, tokens: int, device: str):
    """Routing [T][L][K] and gate inputs [T][L][H] (fp16, CPU) of a batch-1 run with all experts resident, and the
    stack itself (for speculative_guesses; the caller closes it)."""
    gates = [W.gate_weight(shape.seed, l, shape.n_experts, shape.hidden) for l in range(shape.layers)]
    gamma = [W.rms_gamma(shape.hidden) for _ in range(shape.layers)] if shape.rms_eps > 0 else None
    cfgs = [layer_config(shape.hidden, shape.ffn, shape.n_experts, shape.top_k, formats[l][0], formats[l][1],
                         shape.n_experts, 0, shape.rms_eps) for l in range(shape.layers)]
    stack = Stack(cfgs, gates, gamma, n_staging=1, max_batch=1, device=device)
    for l in range(shape.layers):
        for e in range(shape.n_experts):
            mats = W.quantized_expert(shape.seed, l, e, shape.hidden, shape.ffn, formats[l][0], formats[l][1], device)
            for m, mat in enumerate(mats):
                stack.load_expert(l, e, m, *mat)
            del mats
    xs = (W.hidden_iid if shape.hidden_kind == "iid" else W.hidden_ar1)(shape.seed, tokens, 1, shape.hidden)
    xb = [torch.empty(1, shape.hidden, dtype=torch.float16, device=device) for _ in range(2)]
    hb = torch.empty(1, shape.hidden, dtype=torch.float16, device=device)
    routing, h_all = [], torch.empty(tokens, shape.layers, shape.hidden, dtype=torch.float16)
    tr = B.StepTrace()
    for t in range(tokens):
        xb[0].copy_(xs[t])
        torch.cuda.synchronize()
        row = []
        for l in range(shape.layers):
            stack.step_layer(l, xb[l & 1], xb[(l + 1) & 1], hb, tr, prefetch=False)
            stack.synchronize()
            row.append(tr.routing()[0])
            h_all[t, l] = hb[0].cpu()
        routing.append(row)
    return routing, h_all, gates, stack


def speculative_guesses(stack: Stack, h_all: torch.Tensor, ahead: int, m_max: int = B.MOE_MAX_GUESS):
    """guess[t][l] = the m_max most likely experts of layer l+ahead given the gate input of layer l, most likely
    first, as moe_layer_prefetch decides them (every expert of the recording stack is resident, so nothing is
    copied; the decision is reported all the same)."""
    T, L = h_all.shape[0], h_all.shape[1]
    for layer in stack.layers:
        B.moe_layer_set_prefetch(layer, m_max)
    h_dev = h_all.to(stack.device)
    tr = B.StepTrace()
    out = []
    for t in range(T):
        row = []
        for l in range(L - ahead):
            B.moe_layer_prefetch(stack.layers[l + ahead], h_dev[t, l].data_ptr(), 1, tr)
            row.append([tr.guess_expert[i] for i in range(tr.n_guess)])
        out.append(row)
    return out


def lru_hit_ratio(routing, n_layers: int, n_experts: int, top_k: int, k: int) -> float:
    """Replay through the library's cache bookkeeping (host-only context; matrix sizes are irrelevant there)."""
    cfgs = [layer_config(64, 64, n_experts, top_k, 4, 64, k, 0) for _ in range(n_layers)]
    st = Stack(cfgs, [torch.zeros(n_experts, 64) for _ in range(n_layers)], n_staging=1, host_only=True)
    for row in routing:
        for l, sel in enumerate(row):
            B.moe_layer_resolve(st.layers[l], None, list(sel), 1, None, None)
    tot = st.total_stats()
    st.close()
    return tot["hits"] / max(1, tot["needed"])


def speculative_recall_counts(routing, guesses, ahead: int, m: int):
    """(guessed and needed, needed) over all tokens and layers, for the first m of each guess list."""
    got = need = 0
    for t, row in enumerate(guesses):
        for l, g in enumerate(row):
            s = set(routing[t][l + ahead])
            got += len(s.intersection(g[:m]))
            need += len(s)
    return got, need


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="mixtral_stack", choices=sorted(W.CONFIGS))
    ap.add_argument("--tokens", type=int, default=128)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        print("recall_study: no GPU visible", file=sys.stderr)
        return 2
    shape = W.CONFIGS[args.workload]
    formats = W.layer_formats(shape)
    routing, h_all, gates, stack = record(shape, formats, args.tokens, "cuda:0")
    spec = {}
    for a in (1, 2, 10):
        if a >= shape.layers:
            continue
        guesses = speculative_guesses(stack, h_all, a)
        spec[f"{a} ahead"] = {}
        for m in (1, 2, 4):
            got, need = speculative_recall_counts(routing, guesses, a, m)
            spec[f"{a} ahead"][str(m)] = round(got / max(1, need), 4)
    stack.close()
    out = {"workload": shape.name, "tokens": args.tokens, "layers": shape.layers, "experts": shape.n_experts, "top_k": shape.top_k,
           "lru_hit_ratio": {str(k): round(lru_hit_ratio(routing, shape.layers, shape.n_experts, shape.top_k, k), 4)
                             for k in range(shape.top_k, shape.n_experts + 1)},
           "speculative_recall": spec}
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())

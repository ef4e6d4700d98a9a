"""Full-size parity for the 32-layer workloads bench.py times, beyond the headline one (which test_gpu_parity covers):
the mixed 2-bit / 3-bit stack (two blob sizes in one buffer pool, LRU k=4) and the batched 4-bit stack at 16 and 64
tokens per step (matrix cores, 99 MB copies in flight under the staged schedule), plus one prompt-sized step at
Mixtral width.  Every routing decision, cache access and prefetch decision of every (step, layer) is compared with
the oracle; block outputs are compared with the plain-C fp64 oracle on sampled (step, layer, row) points; and the
free-running whole-stack entry point must reproduce the teacher-forced pass bit for bit."""
import numpy as np
import pytest
import torch

import workload as W
from oracle import c_ffn
from oracle import moe_oracle as O
from paper_2312_17238_amd import binding as B

from harness import Model, run_teacher_forced, say

pytestmark = pytest.mark.gpu


def free_running_pass(model: Model, xs: torch.Tensor, outs, tot):
    """The same tokens through moe_stack_step after a reset: bit-identical outputs, the same counters."""
    model.stack.reset()
    dev = model.stack.device
    T, Bn, H = xs.shape
    x_in = torch.empty(Bn, H, dtype=torch.float16, device=dev)
    x_out = torch.empty_like(x_in)
    for t in range(T):
        x_in.copy_(xs[t])
        torch.cuda.synchronize()
        model.stack.step(x_in, x_out, None)
        model.stack.synchronize()
        differ = x_out.cpu().numpy().view(np.uint16) != outs[t].view(np.uint16)
        assert not differ.any(), f"whole-stack step differs at step {t}: {int(differ.sum())} of {differ.size} elements"
    again = model.stack.total_stats()
    for name in ("needed", "hits", "misses", "prefetch_hits", "evictions", "spec_issued", "spec_wasted", "bytes_h2d_demand"):
        assert again[name] == tot[name], name


def test_mixtral_stack_lowbit_full_size():
    """32 layers drawn per layer as 2-bit g16 (88.08 MB blobs) or 3-bit g64 (77.07 MB), LRU k=4, prefetch 2: the
    buffers of the shared pool are sized for the larger blob and hold both kinds side by side.  Decisions on every
    (token, layer) of 17 tokens; the block output in all 32 layers for the first and the seventeenth token."""
    c = W.CONFIGS["mixtral_stack_lowbit"]
    formats = W.layer_formats(c)
    assert {(2, 16), (3, 64)} == set(formats)
    say(f"low-bit stack: build (256 experts; formats {''.join(str(b) for b, _ in formats)})")
    model = Model(c.layers, c.hidden, c.ffn, c.n_experts, c.top_k, formats, c.cache_slots, c.prefetch_m, c.rms_eps,
                  seed=c.seed, keep_layers=[])
    assert sorted(set(model.stack.blob_bytes)) == [77_070_336, 88_080_384]
    T = 17
    xs = W.hidden_ar1(c.seed, T, 1, c.hidden)
    # block outputs: every layer (both formats, every buffer of the pool) for the first token, cold, and for the
    # seventeenth, after the caches have filled
    sampled = {(t, l) for t in (0, 16) for l in range(c.layers)}
    say(f"low-bit stack: teacher-forced run, {len(sampled)} block outputs against the C oracle")
    outs, sim, errs = run_teacher_forced(model, xs, c_ffn.expert_ffn, check_ffn=lambda t, l: (t, l) in sampled)
    assert len(errs) == len(sampled) == 64
    say(f"low-bit stack: max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e}")
    tot = model.stack.total_stats()
    assert tot["needed"] == 2 * T * c.layers
    assert tot["misses"] == sum(s.misses for s in sim.stats) and tot["prefetch_hits"] == sum(s.prefetch_hits for s in sim.stats)
    assert tot["bytes_h2d_demand"] == sum(sim.stats[l].misses * model.stack.blob_bytes[l] for l in range(c.layers))
    free_running_pass(model, xs, outs, tot)
    model.close()


@pytest.mark.parametrize("Bn,T,gemv", [(16, 3, False), (64, 2, False), (4, 3, False), (4, 3, True)])
def test_mixtral_stack_batched_full_size(Bn, T, gemv):
    """32 layers, 4-bit, LRU k=4, prefetch 2, Bn independent streams per step: at 16 and 64 tokens nearly every expert of
    a layer is needed, so a step runs in stages (resident experts first, then the transfers, then the arrivals one by
    one) on the matrix cores with four 99 MB copies in flight per layer; 4 tokens run on the matrix cores too (the
    default from three tokens on) and, with `gemv`, on the GEMV kernels."""
    c = W.CONFIGS["mixtral_stack_batched"]
    say(f"batched stack B={Bn}: build (256 experts)")
    model = Model(c.layers, c.hidden, c.ffn, c.n_experts, c.top_k, None, c.cache_slots, c.prefetch_m, c.rms_eps,
                  max_batch=Bn, seed=c.seed, keep_layers=[])
    B.moe_ctx_profile_enable(model.stack.ctx, True)
    if gemv:
        B.moe_ctx_set_option(model.stack.ctx, "mfma_min_batch", 1000)
    xs = W.hidden_ar1(c.seed, T, Bn, c.hidden)
    # block outputs: three rows of the batch in four layers of the last step (warm cache: hits, misses and confirmed
    # guesses in one step) and two rows in the first layer of the first
    sampled = {(T - 1, l): [0, Bn // 2, Bn - 1] for l in (0, 9, 20, 31)}
    sampled[(0, 0)] = [1, Bn - 2]
    if Bn == 16:                      # and one row in every layer of the last step
        for l in range(c.layers):
            sampled.setdefault((T - 1, l), [5])
    say(f"batched stack B={Bn}: teacher-forced run")
    outs, sim, errs = run_teacher_forced(model, xs, c_ffn.expert_ffn, check_ffn=lambda t, l: (t, l) in sampled,
                                         rows=lambda t, l: sampled[(t, l)])
    assert len(errs) == sum(len(v) for v in sampled.values()) >= 14
    say(f"batched stack B={Bn}: max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e}")
    prof = B.moe_ctx_profile_read(model.stack.ctx).as_dict()
    B.moe_ctx_profile_enable(model.stack.ctx, False)
    assert prof["w13"]["launches"] >= T * c.layers and prof["copy"]["launches"] > 0
    tot = model.stack.total_stats()
    assert tot["needed"] == sum(s.needed for s in sim.stats)
    assert tot["misses"] == sum(s.misses for s in sim.stats) and tot["prefetch_hits"] == sum(s.prefetch_hits for s in sim.stats)
    free_running_pass(model, xs, outs, tot)
    model.close()


def test_mixtral_layer_prompt_sized_step():
    """Prompt encoding at Mixtral width (Sec. 3: the prompt's tokens pass a layer together, each expert loaded once):
    one layer, 384 tokens, LRU k=4 with all 8 experts needed -- three windows of 128 tokens per matrix-core launch,
    rows of 14336 -- every decision, and sampled rows of the block output against the C oracle."""
    c = W.CONFIGS["mixtral_layer"]
    Bn = 384
    say("prompt-sized step at Mixtral width: build")
    model = Model(1, c.hidden, c.ffn, c.n_experts, c.top_k, None, 4, 0, 0.0, max_batch=Bn, seed=c.seed)
    xs = W.hidden_ar1(c.seed, 2, Bn, c.hidden)
    rows = {0: [0, 127, 128, 255, 256, 383], 1: [5, 200, 300]}
    _, sim, errs = run_teacher_forced(model, xs, c_ffn.expert_ffn, rows=lambda t, l: rows[t])
    assert len(errs) == 9
    say(f"prompt-sized step: max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e}")
    st = model.stack.stats()[0]
    assert st["needed"] == 16 and st["misses"] == sim.stats[0].misses >= 8
    model.close()

"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Bit-exact: gate input h, routing indices, cache hit/miss/eviction traces, prefetch
decisions.  Within 2e-2 max-abs / 1e-3 relative RMS: the block output y (fp32, before the residual
add) and x_out.  The comparison is teacher-forced per (token, layer): the oracle recomputes
everything from the fp16 x the engine actually consumed."""
import sys

import numpy as np
import pytest
import torch

import workload as W
from oracle import c_ffn
from oracle import moe_oracle as O
from paper_2312_17238_amd import binding as B
from paper_2312_17238_amd.engine import make_traces

from harness import Model, check_x_out, check_y, oracle_routing, oracle_y, run_teacher_forced, say

pytestmark = pytest.mark.gpu


def test_tiny_layer_every_token():
    """H=256, F=512, 8 experts top-2, 4-bit g64, LRU k=2, 64 i.i.d. tokens, every token checked."""
    c = W.CONFIGS["tiny"]
    say("tiny: build")
    model = Model(1, c.hidden, c.ffn, c.n_experts, c.top_k, None, c.cache_slots, 0, 0.0, seed=c.seed)
    xs = W.hidden_iid(c.seed, c.tokens, 1, c.hidden)
    say("tiny: run")
    _, sim, errs = run_teacher_forced(model, xs, O.expert_ffn)
    st = model.stack.stats()[0]
    assert st["hits"] == sim.stats[0].hits and st["misses"] == sim.stats[0].misses == st["bytes_h2d_demand"] // model.stack.blob_bytes[0]
    assert st["needed"] == 2 * c.tokens
    say(f"tiny: max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e} hits {st['hits']}")
    model.close()


def test_tiny_layer_all_resident_control():
    """Same layer with k = E: after the 8 compulsory misses nothing is ever copied again."""
    c = W.CONFIGS["tiny"]
    model = Model(1, c.hidden, c.ffn, c.n_experts, c.top_k, None, c.n_experts, 0, 0.0, seed=c.seed)
    xs = W.hidden_iid(c.seed, c.tokens, 1, c.hidden)
    run_teacher_forced(model, xs, O.expert_ffn)
    st = model.stack.stats()[0]
    assert st["misses"] == 8 and st["evictions"] == 0 and st["hits"] == 2 * c.tokens - 8
    model.close()


@pytest.mark.parametrize("k,m,Bn,T,gemv", [(2, 2, 1, 40, False), (4, 1, 1, 24, False), (4, 2, 4, 12, False), (4, 2, 4, 12, True),
                                           (4, 2, 16, 8, False), (4, 2, 16, 8, True), (2, 2, 3, 10, False), (2, 2, 3, 10, True)])
def test_small_stack_with_prefetch(k, m, Bn, T, gemv):
    """4 layers, RMSNorm, residual, LRU k, speculative prefetch of m, batch Bn (Bn=16 with k=4 needs
    more experts than slots, so a step runs in several passes).  Batches of three and more tokens run on the matrix
    cores by default; `gemv` keeps them on the GEMV kernels (up to four tokens per expert and launch entry)."""
    L, H, F = 4, 256, 512
    say(f"small stack k={k} m={m} B={Bn} gemv={gemv}: build")
    model = Model(L, H, F, 8, 2, None, k, m, 1e-5, max_batch=Bn, seed=3)
    if gemv:
        B.moe_ctx_set_option(model.stack.ctx, "mfma_min_batch", 1000)
    xs = W.hidden_ar1(3, T, Bn, H)
    say("run")
    outs, sim, errs = run_teacher_forced(model, xs, O.expert_ffn)
    tot = model.stack.total_stats()
    assert tot["prefetch_hits"] == sum(s.prefetch_hits for s in sim.stats)
    assert tot["spec_issued"] == sum(s.spec_issued for s in sim.stats) > 0
    assert tot["spec_wasted"] == sum(s.spec_wasted for s in sim.stats)
    say(f"  recall {(tot['hits'] + tot['prefetch_hits']) / tot['needed']:.3f} prefetch hits {tot['prefetch_hits']} "
        f"max rel-rms {max(e[1] for e in errs):.2e}")
    # the same tokens through the asynchronous whole-stack entry point, after a reset: same traces,
    # bit-identical outputs (Sec. 3.2: prefetching changes no prediction; here also no race changes one)
    model.stack.reset()
    dev = model.stack.device
    x_in = torch.empty(Bn, H, dtype=torch.float16, device=dev)
    x_out = torch.empty(Bn, H, dtype=torch.float16, device=dev)
    sim2 = O.ExpertCacheSim(L, 8, k, 4)
    for t in range(T):
        x_in.copy_(xs[t])
        torch.cuda.synchronize()
        traces = make_traces(L)
        model.stack.step(x_in, x_out, traces)
        model.stack.synchronize()
        assert (x_out.cpu().numpy().view(np.uint16) == outs[t].view(np.uint16)).all(), f"async stack differs at token {t}"
    # and with prefetching off: identical outputs, identical cache contents, only labels and bytes differ
    model.stack.reset()
    model.stack.set_prefetch(0)
    for t in range(T):
        x_in.copy_(xs[t])
        torch.cuda.synchronize()
        model.stack.step(x_in, x_out, None)
        model.stack.synchronize()
        assert (x_out.cpu().numpy().view(np.uint16) == outs[t].view(np.uint16)).all(), f"prefetch-off differs at token {t}"
    off = model.stack.total_stats()
    assert off["prefetch_hits"] == 0 and off["spec_issued"] == 0
    assert off["hits"] == tot["hits"] and off["misses"] == tot["misses"] + tot["prefetch_hits"]
    model.close()


def test_standalone_prefetch_matches_fused_prefetch():
    """moe_layer_prefetch(layer l+1, h_l) takes the decisions step(l, next=l+1) takes."""
    L, H, F = 2, 256, 512
    a = Model(L, H, F, 8, 2, None, 2, 2, 1e-5, seed=5)
    b = Model(L, H, F, 8, 2, None, 2, 2, 1e-5, seed=5)
    xs = W.hidden_ar1(5, 12, 1, H)
    dev = a.stack.device
    x0 = torch.empty(1, H, dtype=torch.float16, device=dev)
    x1 = torch.empty_like(x0); x2 = torch.empty_like(x0); h = torch.empty_like(x0)
    for t in range(xs.shape[0]):
        x0.copy_(xs[t]); torch.cuda.synchronize()
        ta, tb, tp = B.StepTrace(), B.StepTrace(), B.StepTrace()
        a.stack.step_layer(0, x0, x1, None, ta, prefetch=True)
        b.stack.step_layer(0, x0, x1, h, tb, prefetch=False)
        B.moe_layer_prefetch(b.stack.layers[1], h.data_ptr(), 1, tp)
        assert ta.guesses() == tp.guesses() and tb.n_guess == 0
        t1a, t1b = B.StepTrace(), B.StepTrace()
        a.stack.step_layer(1, x1, x2, None, t1a)
        a.stack.synchronize(); ya = x2.cpu().numpy().copy()
        b.stack.step_layer(1, x1, x2, None, t1b)
        b.stack.synchronize()
        assert t1a.accesses() == t1b.accesses() and (ya.view(np.uint16) == x2.cpu().numpy().view(np.uint16)).all()
    assert a.stack.total_stats() == b.stack.total_stats()
    a.close(); b.close()


def test_gate_special_values_and_ties():
    """Equal logits everywhere (zero gate): experts 0 and 1 with weights 1/2; zero input: y = 0."""
    H, F = 256, 512
    from paper_2312_17238_amd.engine import Stack, layer_config
    st = Stack([layer_config(H, F, 8, 2, 4, 64, 2, 0, 1e-5)], [torch.zeros(8, H)], None)
    for e in range(8):
        for mtx, (q, s, z) in enumerate(W.quantized_expert(7, 0, e, H, F, 4, 64)):
            st.load_expert(0, e, mtx, q, s, z)
    dev = st.device
    x = torch.zeros(1, H, dtype=torch.float16, device=dev)
    out = torch.empty_like(x)
    tr = B.StepTrace()
    st.step_layer(0, x, out, None, tr)
    st.synchronize()
    assert tr.routing() == [[0, 1]] and tr.weights() == [[0.5, 0.5]]
    assert (out.cpu().numpy() == 0).all() and (st.read_y(1, H) == 0).all()
    st.close()


def test_mixtral_layer_all_resident():
    """One Mixtral-shaped layer (H=4096, F=14336, 8 experts, 4-bit g64), all experts resident, AR(1) tokens."""
    c = W.CONFIGS["mixtral_layer"]
    say("mixtral layer: build (8 experts of 176M weights)")
    model = Model(1, c.hidden, c.ffn, c.n_experts, c.top_k, None, c.cache_slots, 0, 0.0, seed=c.seed)
    xs = W.hidden_ar1(c.seed, 6, 1, c.hidden)
    say("mixtral layer: run + C oracle")
    _, sim, errs = run_teacher_forced(model, xs, c_ffn.expert_ffn)
    say(f"mixtral layer: max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e}")
    st = model.stack.stats()[0]
    assert st["evictions"] == 0 and st["misses"] <= 8
    model.close()


@pytest.mark.parametrize("path", ["matrix", "gemv"])
def test_mixtral_layer_small_cache_batch4(path):
    """The same shape with k=4 (99 MB demand copies in flight while kernels wait on their events) and batch 4: on the
    matrix cores (the default from three tokens on) and on the GEMV kernels."""
    c = W.CONFIGS["mixtral_layer"]
    say(f"mixtral layer k=4 B=4 {path}: build")
    model = Model(1, c.hidden, c.ffn, c.n_experts, c.top_k, None, 4, 0, 0.0, max_batch=4, seed=c.seed)
    B.moe_ctx_set_option(model.stack.ctx, "mfma_min_batch", 3 if path == "matrix" else 1000)
    xs = W.hidden_ar1(c.seed, 3, 4, c.hidden)
    say("run")
    _, sim, errs = run_teacher_forced(model, xs, c_ffn.expert_ffn, check_ffn=lambda t, l: True)
    say(f"mixtral layer k=4 B=4: max rel-rms {max(e[1] for e in errs):.2e}")
    model.close()


def test_mixtral_stack_full_size_sampled():
    """The headline workload at full size (32 layers, 256 experts of 99 MB in pinned host memory, LRU k=2,
    prefetch m=2, b=4) in the launch configuration bench.py times: routing, cache trace and prefetch decisions
    checked on every (token, layer) of 32 tokens; the block output of every 16th token in all 32 layers against the
    C oracle."""
    c = W.CONFIGS["mixtral_stack"]
    say("mixtral stack: build (256 experts)")
    model = Model(c.layers, c.hidden, c.ffn, c.n_experts, c.top_k, None, c.cache_slots, c.prefetch_m, c.rms_eps,
                  seed=c.seed, keep_layers=[])
    T = 32
    xs = W.hidden_ar1(c.seed, T, 1, c.hidden)
    say("mixtral stack: teacher-forced run, block output of every 16th token checked in every layer")
    outs, sim, errs = run_teacher_forced(model, xs, c_ffn.expert_ffn, check_ffn=lambda t, l: t % 16 == 0)
    assert len(errs) == 2 * c.layers
    say(f"mixtral stack: max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e}")
    tot = model.stack.total_stats()
    assert tot["needed"] == 2 * T * c.layers
    assert tot["misses"] == sum(s.misses for s in sim.stats) and tot["prefetch_hits"] == sum(s.prefetch_hits for s in sim.stats)
    # the same tokens through the asynchronous stack entry point (what bench.py calls): bit-identical outputs
    model.stack.reset()
    dev = model.stack.device
    x_in = torch.empty(1, c.hidden, dtype=torch.float16, device=dev)
    x_out = torch.empty_like(x_in)
    for t in range(T):
        x_in.copy_(xs[t])
        torch.cuda.synchronize()
        model.stack.step(x_in, x_out, None)
        model.stack.synchronize()
        assert (x_out.cpu().numpy().view(np.uint16) == outs[t].view(np.uint16)).all(), f"async stack differs at token {t}"
    assert model.stack.total_stats() == tot
    # ... and with bench.py's default of speculative loads as a 4 MiB head plus a confirmed tail: the same outputs and
    # decisions, fewer bytes for the wrong guesses
    model.stack.reset()
    B.moe_ctx_set_option(model.stack.ctx, "spec_head_mb", 4)
    for t in range(T):
        x_in.copy_(xs[t])
        torch.cuda.synchronize()
        model.stack.step(x_in, x_out, None)
        model.stack.synchronize()
        assert (x_out.cpu().numpy().view(np.uint16) == outs[t].view(np.uint16)).all(), f"head-then-tail stack differs at token {t}"
    tot4 = model.stack.total_stats()
    for key in ("needed", "hits", "prefetch_hits", "misses", "evictions", "spec_issued", "spec_wasted", "bytes_h2d_demand"):
        assert tot4[key] == tot[key], key
    blob = model.stack.blob_bytes[0]
    assert tot4["bytes_h2d_spec"] == tot["bytes_h2d_spec"] - tot["spec_wasted"] * (blob - (4 << 20))
    model.close()


@pytest.mark.parametrize("formats,Bn", [([(2, 16)] * 3, 1), ([(3, 64)] * 3, 1), ([(2, 16), (3, 64), (4, 64)], 1),
                                        ([(3, 64), (2, 16), (4, 32)], 4), ([(4, 128), (3, 64), (2, 16)], 2)])
def test_small_stack_low_bit_formats(formats, Bn):
    """2-bit g16 and 3-bit g64 experts (and other 4-bit group sizes), formats mixed per layer so the shared
    buffer pool holds blobs of different sizes; LRU k=4, prefetch 2."""
    L, H, F = len(formats), 256, 512
    say(f"low-bit stack {formats} B={Bn}")
    model = Model(L, H, F, 8, 2, formats, 4, 2, 1e-5, max_batch=Bn, seed=21)
    xs = W.hidden_ar1(21, 16, Bn, H)
    _, sim, errs = run_teacher_forced(model, xs, O.expert_ffn)
    say(f"  max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e}")
    model.close()


@pytest.mark.parametrize("bits,group", [(2, 16), (3, 64)])
def test_mixtral_layer_low_bit(bits, group):
    """One Mixtral-shaped layer with 2-bit g16 / 3-bit g64 experts, k=4, C oracle on every token."""
    c = W.CONFIGS["mixtral_layer"]
    say(f"mixtral layer {bits}-bit g{group}: build")
    model = Model(1, c.hidden, c.ffn, c.n_experts, c.top_k, [(bits, group)], 4, 0, 0.0, seed=c.seed)
    xs = W.hidden_ar1(c.seed, 4, 1, c.hidden)
    _, sim, errs = run_teacher_forced(model, xs, c_ffn.expert_ffn)
    say(f"  max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e}")
    model.close()


@pytest.mark.parametrize("formats", [[(4, 64)] * 2, [(3, 64), (2, 16)]])
def test_single_token_kernel_variants_agree(formats):
    """A single-token step has three implementations: the general kernels (atomics + residual kernel), the
    w2 kernel with in-kernel combine and residual (default), and one persistent launch with a grid barrier.
    All three must give bit-identical outputs, traces and statistics."""
    L, H, F = len(formats), 256, 512
    xs = W.hidden_ar1(31, 24, 1, H)
    outs = {}
    for name, token_path, fused in (("general", 0, 0), ("token", 1, 0), ("one_launch", 1, 1), ("one_launch_seq", 1, 2)):
        model = Model(L, H, F, 8, 2, formats, 2, 2, 1e-5, seed=31)
        B.moe_ctx_set_option(model.stack.ctx, "token_path", token_path)
        B.moe_ctx_set_option(model.stack.ctx, "fused", fused)
        B.moe_ctx_profile_enable(model.stack.ctx, True)
        o, sim, errs = run_teacher_forced(model, xs, O.expert_ffn)
        prof = B.moe_ctx_profile_read(model.stack.ctx).as_dict()
        assert (prof["ffn"]["launches"] > 0) == name.startswith("one_launch")
        assert (prof["w13"]["launches"] > 0) == (not name.startswith("one_launch"))
        outs[name] = (o, model.stack.total_stats())
        model.close()
    for other in ("token", "one_launch", "one_launch_seq"):
        for a, b in zip(outs["general"][0], outs[other][0]):
            assert (a.view(np.uint16) == b.view(np.uint16)).all(), other
        assert outs["general"][1] == outs[other][1]


@pytest.mark.parametrize("Bn,token_path", [(1, 1), (1, 0), (3, 1)])
def test_launch_shape_knobs_do_not_change_results(Bn, token_path):
    """The tuning knobs (blocks of the w1/w3 kernel, rows per block of the two w2 kernels, waiting for the gate with
    a stream synchronisation instead of polling) only move work between blocks: outputs, traces and statistics
    stay bit-identical, also for odd values that leave ragged last blocks."""
    L, H, F = 2, 256, 512
    xs = W.hidden_ar1(37, 12, Bn, H)
    outs = []
    for knobs in ({}, {"w13_blocks": 7, "w2_rows": 5, "w2_token_rows": 3, "sync_wait": 1}, {"w13_blocks": 1000, "w2_rows": 64, "w2_token_rows": 64}):
        model = Model(L, H, F, 8, 2, [(4, 64), (3, 64)], 2, 2, 1e-5, max_batch=Bn, seed=37)
        B.moe_ctx_set_option(model.stack.ctx, "mfma_min_batch", 1000)      # the knobs are the GEMV kernels'
        B.moe_ctx_set_option(model.stack.ctx, "token_path", token_path)
        for name, value in knobs.items():
            B.moe_ctx_set_option(model.stack.ctx, name, value)
        o, sim, errs = run_teacher_forced(model, xs, O.expert_ffn)
        outs.append((o, model.stack.total_stats()))
        model.close()
    for o, st in outs[1:]:
        for a, b in zip(outs[0][0], o):
            assert (a.view(np.uint16) == b.view(np.uint16)).all()
        assert st == outs[0][1]


@pytest.mark.parametrize("form", [3, 2, 1, 4, 5])
@pytest.mark.parametrize("Bn,k", [(16, 4), (64, 4), (33, 8), (64, 2)])
def test_small_stack_matrix_core_path(Bn, k, form):
    """Batches of 16 and more run 4-bit g64 experts as grouped dequantize+GEMM on the matrix cores
    (more than 32 tokens on one expert needs two token tiles; k=2 with 8 needed experts needs several passes).
    All kernel forms (3: fp16 weights from one fma plus a rank-1 correction, the default; 2: fp16 weights with the exact subtraction; 1: fp32 group scaling) meet the same bound against the oracle."""
    L, H, F = 3, 256, 512
    say(f"matrix-core stack B={Bn} k={k} form={form}")
    model = Model(L, H, F, 8, 2, None, k, 2, 1e-5, max_batch=Bn, seed=41)
    B.moe_ctx_set_option(model.stack.ctx, "mfma_form", form)
    B.moe_ctx_set_option(model.stack.ctx, "mfma16_waves", 8 if k == 4 else 4)
    B.moe_ctx_profile_enable(model.stack.ctx, True)
    xs = W.hidden_ar1(41, 5, Bn, H)
    _, sim, errs = run_teacher_forced(model, xs, O.expert_ffn)
    say(f"  max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e}")
    model.close()


@pytest.mark.parametrize("form,rel", [(1, 1e-4), (2, 2e-3), (3, 2e-3), (4, 2e-3), (5, 1e-4)])
def test_matrix_core_path_agrees_with_gemv_path(form, rel):
    """The same batched steps through the GEMV kernels (threshold raised) and the matrix cores: identical
    traces; outputs equal to within the summation-order noise of fp32 for the form that scales groups in fp32,
    and to within the rounding of the weights to fp16 for the form that dequantises before the multiply."""
    L, H, F, Bn = 2, 256, 512, 24
    xs = W.hidden_ar1(43, 4, Bn, H)
    res = {}
    for name, thr in (("gemv", 1000), ("mfma", 1)):
        model = Model(L, H, F, 8, 2, None, 4, 2, 1e-5, max_batch=Bn, seed=43)
        B.moe_ctx_set_option(model.stack.ctx, "mfma_min_batch", thr)
        B.moe_ctx_set_option(model.stack.ctx, "mfma_form", form)
        dev = model.stack.device
        x_in = torch.empty(Bn, H, dtype=torch.float16, device=dev); x_out = torch.empty_like(x_in)
        ys = []
        x_in.copy_(xs[0]); torch.cuda.synchronize()
        tr = B.StepTrace()
        model.stack.step_layer(0, x_in, x_out, None, tr)
        model.stack.synchronize()
        res[name] = (model.stack.read_y(Bn, H).copy(), tr.accesses(), tr.routing())
        model.close()
    assert res["gemv"][1:] == res["mfma"][1:]
    d = np.abs(res["gemv"][0] - res["mfma"][0]).max()
    say(f"matrix cores form {form} vs gemv: max abs diff {d:.3e} of max {np.abs(res['gemv'][0]).max():.3e}")
    assert d < rel * max(1.0, np.abs(res["gemv"][0]).max()), d


@pytest.mark.parametrize("form", [3, 4, 5])
@pytest.mark.parametrize("Bn,T,k", [(16, 2, 4), (64, 1, 8)])
def test_mixtral_layer_batch16_matrix_cores(Bn, T, k, form):
    """Mixtral-shaped layer on the matrix cores, C oracle on every row: batch 16 with k=4 (8 needed experts over 4
    slots: several passes) and batch 64 with every expert resident (the launch shape bench.py times for the kernels)."""
    c = W.CONFIGS["mixtral_layer"]
    say(f"mixtral layer B={Bn} k={k} matrix cores: build")
    model = Model(1, c.hidden, c.ffn, c.n_experts, c.top_k, None, k, 0, 0.0, max_batch=Bn, seed=c.seed)
    B.moe_ctx_set_option(model.stack.ctx, "mfma_form", form)
    B.moe_ctx_set_option(model.stack.ctx, "mfma16_waves", 8)
    xs = W.hidden_ar1(c.seed, T, Bn, c.hidden)
    _, sim, errs = run_teacher_forced(model, xs, c_ffn.expert_ffn)
    say(f"  form {form}: max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e}")
    model.close()


@pytest.mark.parametrize("form", [5, 2])
@pytest.mark.parametrize("Bn,k", [(16, 8), (64, 8)])
def test_mixtral_layer_two_level_metadata_matrix_cores(Bn, k, form):
    """Mixtral-shaped layer with two-level metadata (scale group 128: one run per row of w1/w3, two per row of w2) on
    the matrix cores, one and two token tiles, C oracle on every row: the group-scaled kernels decode scale and zero
    in fp32 (default), form 2 dequantises to fp16 first."""
    c = W.CONFIGS["mixtral_layer"]
    say(f"mixtral layer, two-level metadata, B={Bn} form {form}: build")
    model = Model(1, c.hidden, c.ffn, c.n_experts, c.top_k, None, k, 0, 0.0, max_batch=Bn, seed=c.seed, scale_group=128)
    B.moe_ctx_set_option(model.stack.ctx, "mfma_form", form)
    xs = W.hidden_ar1(c.seed, 1, Bn, c.hidden)
    _, sim, errs = run_teacher_forced(model, xs, c_ffn.expert_ffn)
    say(f"  form {form}: max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e}")
    model.close()


def test_rmsnorm_small_and_large_inputs_bit_exact():
    """eps dominates for tiny inputs and the straight fp64->fp16 rounding matters for large ones: h must equal
    the oracle's bit for bit over magnitudes from fp16 subnormals to near overflow."""
    from paper_2312_17238_amd.engine import Stack, layer_config
    H, F = 256, 512
    gate = W.gate_weight(9, 0, 8, H)
    st = Stack([layer_config(H, F, 8, 2, 4, 64, 8, 0, 1e-5)], [gate], None, max_batch=8)
    for e in range(8):
        for mtx, (q, s, z) in enumerate(W.quantized_expert(9, 0, e, H, F, 4, 64)):
            st.load_expert(0, e, mtx, q, s, z)
    base = W.hidden_iid(9, 1, 8, H)[0].float()
    scales = torch.tensor([2.0 ** -20, 2.0 ** -12, 2.0 ** -8, 2.0 ** -4, 1.0, 16.0, 1024.0, 12000.0]).unsqueeze(1)
    x = (base * scales).clamp(-60000, 60000).to(torch.float16)
    dev = st.device
    xd = x.to(dev); out = torch.empty_like(xd); h = torch.empty_like(xd)
    tr = B.StepTrace()
    st.step_layer(0, xd, out, h, tr)
    st.synchronize()
    gam = np.ones(H, np.float16)
    want = O.rmsnorm(x.numpy(), gam, 1e-5)
    assert (h.cpu().numpy().view(np.uint16) == want.view(np.uint16)).all()
    for b in range(8):
        idx, w, z = O.route(gate.numpy(), want[b], 2)
        assert tr.routing()[b] == idx
    st.close()


def test_speculative_head_then_tail_is_invisible_in_results():
    """Option spec_head_mb: a speculative load moves only the head of the expert and the rest once the guess is
    confirmed.  Decisions, traces, statistics (except bytes) and outputs must be identical to whole-expert loads."""
    c = W.CONFIGS["mixtral_layer"]
    L, T = 3, 6
    xs = W.hidden_ar1(51, T, 1, c.hidden)
    res = {}
    for head in (0, 8):
        model = Model(L, c.hidden, c.ffn, 8, 2, None, 2, 2, 1e-5, seed=51, keep_layers=[])
        B.moe_ctx_set_option(model.stack.ctx, "spec_head_mb", head)
        outs, sim, errs = run_teacher_forced(model, xs, c_ffn.expert_ffn, check_ffn=lambda t, l: (t, l) in {(1, 1), (4, 2)})
        res[head] = (outs, model.stack.total_stats())
        model.close()
    for a, b in zip(res[0][0], res[8][0]):
        assert (a.view(np.uint16) == b.view(np.uint16)).all()
    s0, s8 = res[0][1], res[8][1]
    for k in s0:
        if k != "bytes_h2d_spec":
            assert s0[k] == s8[k], k
    blob = B.moe_expert_blob_bytes(c.hidden, c.ffn, 4, 64)
    assert s0["bytes_h2d_spec"] == s0["spec_issued"] * blob
    assert s8["bytes_h2d_spec"] == s8["spec_issued"] * (8 << 20) + s8["prefetch_hits"] * (blob - (8 << 20))
    assert s8["prefetch_hits"] > 0 and s8["spec_wasted"] > 0


@pytest.mark.parametrize("E,K,k,m,Bn,T,path", [
    (16, 4, 4, 4, 64, 3, "gemv"),      # every limit of the ABI at once: 16 experts, top-4, 4 guesses, batch 64 (256 pairs)
    (16, 4, 4, 4, 64, 3, "matrix"),    # the same through the matrix cores (up to 16 needed experts over 4 slots: 4 passes)
    (16, 4, 16, 2, 17, 3, "matrix"),   # all 16 resident, ragged batch
    (2, 2, 2, 2, 1, 8, "gemv"),        # top_k = E: both experts always selected, the gate only sets the weights
    (4, 1, 1, 1, 2, 8, "gemv"),        # top-1 with a single slot: every change of expert is a miss
    (3, 2, 3, 0, 5, 4, "gemv"),        # odd expert count, no speculation, batch between the GEMV chunk sizes
])
def test_limits_and_degenerate_shapes(E, K, k, m, Bn, T, path):
    """The extremes the interface allows (MOE_MAX_EXPERTS, MOE_MAX_TOPK, MOE_MAX_GUESS, MOE_MAX_BATCH) and the
    degenerate shapes of the method, every decision and every output row checked against the oracle."""
    L, H, F = 3, 256, 512
    say(f"limits E={E} K={K} k={k} m={m} B={Bn} {path}")
    model = Model(L, H, F, E, K, None, k, m, 1e-5, max_batch=Bn, seed=51)
    B.moe_ctx_set_option(model.stack.ctx, "mfma_min_batch", 16 if path == "matrix" else 1000)
    B.moe_ctx_profile_enable(model.stack.ctx, True)
    xs = W.hidden_ar1(51, T, Bn, H)
    _, sim, errs = run_teacher_forced(model, xs, O.expert_ffn)
    prof = B.moe_ctx_profile_read(model.stack.ctx).as_dict()
    assert prof["w13"]["launches"] > 0
    tot = model.stack.total_stats()
    assert tot["needed"] == sum(s.needed for s in sim.stats)
    assert tot["misses"] == sum(s.misses for s in sim.stats)
    say(f"  max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e} misses {tot['misses']}")
    model.close()


def test_largest_supported_matrices():
    """H = 8192, F = 16384 (the largest shapes the kernels accept: four 2048-code chunks per w1/w3 row, eight per w2
    row), two experts, one token at a time, C oracle on every row."""
    H, F = 8192, 16384
    say("largest matrices: build")
    model = Model(1, H, F, 2, 2, None, 2, 0, 1e-5, seed=53)
    xs = W.hidden_ar1(53, 2, 1, H)
    say("largest matrices: run")
    _, sim, errs = run_teacher_forced(model, xs, c_ffn.expert_ffn)
    say(f"  max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e}")
    model.close()


@pytest.mark.parametrize("H,F,k,m,Bn,T,head_mb", [(256, 512, 2, 2, 1, 48, 0), (1024, 2048, 2, 2, 1, 20, 1), (256, 512, 4, 2, 4, 12, 0),
                                                  (256, 512, 4, 2, 16, 6, 0), (256, 512, 2, 1, 8, 6, 0), (256, 512, 4, 2, 100, 5, 0), (256, 512, 2, 2, 80, 4, 0)])
def test_swap_eviction_keeps_every_expert_intact(H, F, k, m, Bn, T, head_mb):
    """Sec. 3.3, hosts that cannot hold every expert (MOE_LAYER_SWAP): every load writes the evicted expert back
    to the host.  Over many swaps every decision still equals the oracle's, every expert sits where the oracle's
    placement says, every output row is in tolerance (a blob damaged on its way out or back would show as soon as
    the expert is used again), and the outputs are bit-identical to the same stack without swapping.  The 3.5 MB
    blobs of the H=1024 case with a 1 MiB head also cover a confirmed guess whose tail is read from the host buffer
    the expert is about to vacate.  Batches above 64 tokens take the prompt-sized schedule (resident experts first,
    transfers into their buffers guarded by that launch)."""
    L, E = 4, 8
    xs = W.hidden_ar1(61, T, Bn, H)
    outs = {}
    for name, flags in (("swap", B.MOE_LAYER_SWAP), ("plain", 0)):
        say(f"swap eviction k={k} m={m} B={Bn} head={head_mb} MiB: {name}")
        model = Model(L, H, F, E, 2, None, k, m, 1e-5, max_batch=Bn, seed=61, init_policy=1, flags=flags)
        B.moe_ctx_set_option(model.stack.ctx, "spec_head_mb", head_mb)
        sim = O.ExpertCacheSim(L, E, k, 4, warm=True)
        place = [O.SwapPlacement(E, k) for _ in range(L)] if flags else None
        o, sim, errs = run_teacher_forced(model, xs, O.expert_ffn, sim=sim, placement=place)
        tot = model.stack.total_stats()
        blob = model.stack.blob_bytes[0]
        if flags:
            assert tot["bytes_d2h_writeback"] == sum(p.writebacks for p in place) * blob == tot["evictions"] * blob > 0
        else:
            assert tot["bytes_d2h_writeback"] == 0
        outs[name] = (o, {n: v for n, v in tot.items() if n != "bytes_d2h_writeback"})
        say(f"  max rel-rms {max(e[1] for e in errs):.2e} evictions {tot['evictions']}")
        model.close()
    for a, b in zip(outs["swap"][0], outs["plain"][0]):
        assert (a.view(np.uint16) == b.view(np.uint16)).all()
    assert outs["swap"][1] == outs["plain"][1]


def test_swap_eviction_mixtral_layer():
    """One Mixtral-shaped layer in swap mode, k=2: 99 MB blobs travel both ways; C oracle on every token."""
    c = W.CONFIGS["mixtral_layer"]
    say("swap eviction, mixtral layer: build")
    model = Model(1, c.hidden, c.ffn, c.n_experts, c.top_k, None, 2, 0, 0.0, seed=c.seed, init_policy=1, flags=B.MOE_LAYER_SWAP)
    xs = W.hidden_ar1(c.seed, 12, 1, c.hidden)
    sim = O.ExpertCacheSim(1, c.n_experts, 2, 4, warm=True)
    place = [O.SwapPlacement(c.n_experts, 2)]
    _, sim, errs = run_teacher_forced(model, xs, c_ffn.expert_ffn, sim=sim, placement=place)
    st = model.stack.stats()[0]
    assert st["bytes_d2h_writeback"] == st["misses"] * model.stack.blob_bytes[0] > 0
    say(f"  max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e} write-backs {place[0].writebacks}")
    model.close()


def test_two_level_metadata_several_runs_on_the_matrix_cores():
    """H=1024 and F=2048 give 16 and 32 groups per row; with runs of 8 groups a row has 2 and 4 runs, each of them one
    step of the streaming matrix-core kernel."""
    model = Model(2, 1024, 2048, 8, 2, None, 4, 2, 1e-5, max_batch=24, seed=73, scale_group=8)
    B.moe_ctx_profile_enable(model.stack.ctx, True)
    xs = W.hidden_ar1(73, 3, 24, 1024)
    _, sim, errs = run_teacher_forced(model, xs, O.expert_ffn)
    say(f"two-level, runs of 8, matrix cores: max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e}")
    model.close()


@pytest.mark.parametrize("R,Bn,k,m,variant", [(256, 1, 2, 2, "token"), (2, 1, 2, 2, "token"), (2, 1, 2, 1, "general"), (2, 1, 2, 2, "one_launch"),
                                              (2, 4, 4, 2, "general"), (256, 16, 4, 2, "matrix"), (2, 40, 4, 2, "matrix"),
                                              (4, 200, 2, 1, "matrix"), (4, 3, 8, 0, "general"), (2, 20, 4, 2, "gemv")])
def test_small_stack_two_level_metadata(R, Bn, k, m, variant):
    """4-bit experts whose scales and zeros are themselves 8-bit codes (Sec. 4.2 "scale group size"): runs of R groups
    per row (R=2 gives 2 and 4 runs per row here, R=256 one), through the single-token kernels, the general GEMV
    kernels, the one-launch kernel, and batches on the matrix cores (and on the GEMV kernels, threshold raised)."""
    L, H, F = 3, 256, 512
    say(f"two-level metadata R={R} B={Bn} k={k} m={m} {variant}")
    model = Model(L, H, F, 8, 2, None, k, m, 1e-5, max_batch=Bn, seed=71, scale_group=R)
    B.moe_ctx_set_option(model.stack.ctx, "token_path", 0 if variant == "general" else 1)
    B.moe_ctx_set_option(model.stack.ctx, "fused", 1 if variant == "one_launch" else 0)
    B.moe_ctx_set_option(model.stack.ctx, "mfma_min_batch", 1000 if variant == "gemv" else 16)
    assert model.stack.blob_bytes[0] == B.moe_expert_blob_bytes(H, F, 4, 64, R)
    xs = W.hidden_ar1(71, 10 if Bn < 100 else 2, Bn, H)
    _, sim, errs = run_teacher_forced(model, xs, O.expert_ffn)
    say(f"  max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e}")
    model.close()


@pytest.mark.parametrize("formats,R,F,Bn,k,m,variant", [
    ([(3, 64)] * 3, 2, 448, 1, 2, 2, "token"), ([(3, 64)] * 3, 4, 448, 1, 2, 1, "general"), ([(3, 64)] * 3, 128, 448, 1, 4, 2, "token"),
    ([(2, 16)] * 3, 4, 320, 1, 2, 2, "token"), ([(2, 16)] * 3, 8, 320, 1, 2, 1, "general"), ([(2, 16)] * 3, 128, 320, 1, 4, 2, "token"),
    ([(2, 16), (3, 64), (2, 16)], 8, 448, 4, 4, 2, "general"), ([(3, 64), (2, 16), (3, 64)], 4, 320, 20, 4, 2, "general"),
    ([(2, 16), (3, 64), (4, 64)], 8, 448, 2, 8, 0, "general")])
def test_small_stack_two_level_metadata_low_bit(formats, R, F, Bn, k, m, variant):
    """The 3-bit g64 and 2-bit g16 schemes with 8-bit scale and zero codes (Sec. 4.2 pairs both with scale group size
    128).  H=256 gives 4 (16 for 2-bit) groups per w1/w3 row; F=448 gives 7 groups of 64 (runs of 2: 2+2+2+1, of 4: 4+3)
    and 28 of 16 (runs of 8: 8+8+8+4); F=320 gives 5 and 20 (runs of 8: 8+8+4): rows that end in a shorter run, several
    runs per row, whole rows as one run, through the single-token and the general kernels with 1, 2 and 4 tokens
    per entry."""
    L, H = 3, 256
    say(f"two-level metadata low-bit formats={formats} R={R} F={F} B={Bn} k={k} m={m} {variant}")
    model = Model(L, H, F, 8, 2, formats, k, m, 1e-5, max_batch=Bn, seed=79, scale_group=R)
    B.moe_ctx_set_option(model.stack.ctx, "token_path", 0 if variant == "general" else 1)
    for l, (bits, g) in enumerate(formats):
        assert model.stack.blob_bytes[l] == B.moe_expert_blob_bytes(H, F, bits, g, R)
    xs = W.hidden_ar1(79, 10 if Bn < 10 else 4, Bn, H)
    _, sim, errs = run_teacher_forced(model, xs, O.expert_ffn)
    say(f"  max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e}")
    model.close()


@pytest.mark.parametrize("bits,g,blob", [(3, 64, 72_089_600), (2, 16, 66_781_184)])
def test_mixtral_layer_two_level_metadata_low_bit(bits, g, blob):
    """One Mixtral-shaped layer in the paper's 3-bit and 2-bit schemes with scale group 128 (w2 rows of the 3-bit
    scheme: 224 groups = one run of 128 and one of 96), k=4, C oracle on every token."""
    c = W.CONFIGS["mixtral_layer"]
    say(f"mixtral layer, {bits}-bit g{g}, scale group 128: build")
    model = Model(1, c.hidden, c.ffn, c.n_experts, c.top_k, [(bits, g)], 4, 0, 0.0, seed=c.seed, scale_group=128)
    assert model.stack.blob_bytes[0] == blob
    xs = W.hidden_ar1(c.seed, 5, 1, c.hidden)
    _, sim, errs = run_teacher_forced(model, xs, c_ffn.expert_ffn)
    say(f"  max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e}")
    model.close()


def test_mixtral_layer_two_level_metadata():
    """One Mixtral-shaped layer with two-level metadata (scale group 256: one run per row), k=4, C oracle on every token."""
    c = W.CONFIGS["mixtral_layer"]
    say("mixtral layer, two-level metadata: build")
    model = Model(1, c.hidden, c.ffn, c.n_experts, c.top_k, None, 4, 0, 0.0, seed=c.seed, scale_group=256)
    assert model.stack.blob_bytes[0] == 94_109_696
    xs = W.hidden_ar1(c.seed, 6, 1, c.hidden)
    _, sim, errs = run_teacher_forced(model, xs, c_ffn.expert_ffn)
    say(f"  max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e}")
    model.close()


@pytest.mark.parametrize("formats,scale_group,init_policy,m", [([(4, 64)] * 3, 0, 0, 2), ([(4, 64)] * 3, 0, 1, 0), ([(2, 16), (3, 64), (4, 64)], 0, 1, 2),
                                                               ([(4, 64), (3, 64), (2, 16)], 8, 0, 1)])
def test_device_routed_steps_against_oracle_and_waiting_steps(formats, scale_group, init_policy, m):
    """A layer with every expert resident (k = E) takes single-token steps without the host waiting for the gate:
    the FFN kernels read the selection the gate kernel left on the device, the cache bookkeeping is caught up later.
    Checked against the oracle (gate input bit-exact, y within tolerance, the cache simulator's counters and
    recency order at the end) and against the same run with the feature off (outputs bit-identical, counters and
    stamps equal), from a cold start (the first steps still wait, until every slot is filled) and from a warm one,
    with a waiting step (one that asks for a trace) thrown in every few tokens."""
    L, H, F, E, K, T = 3, 256, 512, 8, 2, 40
    say(f"device-routed steps formats={formats} scale_group={scale_group} init_policy={init_policy} m={m}")
    fast = Model(L, H, F, E, K, formats, E, m, 1e-5, seed=91, init_policy=init_policy, scale_group=scale_group)
    slow = Model(L, H, F, E, K, formats, E, m, 1e-5, seed=91, init_policy=init_policy, scale_group=scale_group, keep_layers=[])
    B.moe_ctx_set_option(slow.stack.ctx, "device_routing", 0)
    xs = W.hidden_ar1(91, T, 1, H)
    dev = fast.stack.device
    sim = O.ExpertCacheSim(L, E, E, 4, warm=(init_policy == 1))
    xa = [torch.empty(1, H, dtype=torch.float16, device=dev) for _ in range(L + 1)]
    xb = [torch.empty(1, H, dtype=torch.float16, device=dev) for _ in range(L + 1)]
    hb = torch.empty(1, H, dtype=torch.float16, device=dev)
    errs = []
    for t in range(T):
        xa[0].copy_(xs[t]); xb[0].copy_(xs[t])
        torch.cuda.synchronize()
        for l in range(L):
            tr = B.StepTrace() if t % 7 == 3 else None
            fast.stack.step_layer(l, xa[l], xa[l + 1], hb, tr)
            slow.stack.step_layer(l, xb[l], xb[l + 1], None, None)
            fast.stack.synchronize(); slow.stack.synchronize()
            x_np = xa[l].cpu().numpy()
            (h, idx, w, _), = oracle_routing(fast, l, x_np)
            assert (hb.cpu().numpy()[0].view(np.uint16) == h.view(np.uint16)).all(), f"gate input differs t={t} l={l}"
            guess = O.prefetch_guess(O.prefetch_scores(fast.gate_np(l + 1), h[None]), m) if (l + 1 < L and m > 0) else None
            sim.step(l, [idx], guess)
            y_ref = oracle_y(fast, l, h, idx, w, O.expert_ffn)
            errs.append(check_y(fast.stack.read_y(1, H)[0], y_ref, f"y t={t} l={l}"))
            assert (xa[l + 1].cpu().numpy().view(np.uint16) == xb[l + 1].cpu().numpy().view(np.uint16)).all(), f"x_out differs t={t} l={l}"
    sa, sb = fast.stack.stats(), slow.stack.stats()
    routed = [d.pop("steps_device_routed") for d in sa]
    assert all(d.pop("steps_device_routed") == 0 for d in sb) and sa == sb
    # every step without a trace is device-routed once the layer (and, with speculation, the next one) is full
    traced = len([t for t in range(T) if t % 7 == 3])
    say(f"  device-routed steps per layer: {routed} of {T} ({traced} asked for a trace)")
    assert all(0 < r <= T - traced for r in routed) and (init_policy == 0 or all(r == T - traced for r in routed))
    for l in range(L):
        assert sa[l]["hits"] == sim.stats[l].hits and sa[l]["misses"] == sim.stats[l].misses and sa[l]["steps"] == T
        ca, cb = B.moe_layer_cache_state(fast.stack.layers[l], E), B.moe_layer_cache_state(slow.stack.layers[l], E)
        assert ca == cb
        # recency order of the slots = the simulator's
        order = [e for _, e in sorted(zip(ca[1], ca[0]))]
        assert order == [e for _, e in sorted(zip(sim.slot_stamp[l], sim.slot_expert[l]))]
    say(f"  max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e}")
    fast.close(); slow.close()


def test_device_routed_steps_log_wraps():
    """More device-routed steps than the selection log has entries, with no call in between that would catch the
    bookkeeping up: the library does it by itself when the log is full, and the counters come out complete."""
    H, F, E, T = 256, 512, 8, 9000
    model = Model(1, H, F, E, 2, None, E, 0, 0.0, seed=93, init_policy=1, keep_layers=[])
    xs = W.hidden_iid(93, 64, 1, H).to(model.stack.device)
    x_out = torch.empty(1, H, dtype=torch.float16, device=model.stack.device)
    for t in range(T):
        model.stack.step(xs[t % 64], x_out, None)
    model.stack.synchronize()
    st = model.stack.stats()[0]
    assert st["steps"] == T == st["steps_device_routed"] and st["needed"] == 2 * T == st["hits"] and st["misses"] == 0
    model.close()


def test_profile_timeline_matches_profile_totals():
    """The diagnostic timeline lists every timed launch of a kind with start <= stop, in issue order, and its
    durations add up to what moe_ctx_profile_read reports; with a copy stride of 3 a third of the transfers is timed."""
    model = Model(3, 256, 512, 8, 2, None, 2, 2, 1e-5, seed=97, keep_layers=[])
    B.moe_ctx_set_option(model.stack.ctx, "profile_copy_stride", 3)
    B.moe_ctx_profile_enable(model.stack.ctx, True)
    xs = W.hidden_ar1(97, 12, 1, 256).to(model.stack.device)
    x_out = torch.empty(1, 256, dtype=torch.float16, device=model.stack.device)
    for t in range(12):
        model.stack.step(xs[t], x_out, None)
    model.stack.synchronize()
    lines = {k: B.moe_ctx_profile_timeline(model.stack.ctx, k) for k in range(6)}
    prof = B.moe_ctx_profile_read(model.stack.ctx).as_dict()
    for k, name in enumerate(("gate", "w13", "w2", "copy", "ffn", "writeback")):
        tl = lines[k]
        assert len(tl) == prof[name]["launches"]
        assert all(0.0 <= a <= b for a, b in tl) and all(tl[i][0] <= tl[i + 1][0] for i in range(len(tl) - 1))
        assert abs(sum(b - a for a, b in tl) - prof[name]["total_ms"]) <= 1e-3 * max(1.0, prof[name]["total_ms"])
    st = model.stack.total_stats()
    n_copies = st["misses"] + st["spec_issued"]
    assert len(lines[0]) == len(lines[1]) == len(lines[2]) == 36 and len(lines[3]) == -(-n_copies // 3) and not lines[4] and not lines[5]
    model.close()


def test_recall_study_tool_against_closed_forms_and_oracle():
    """paper_2312_17238_amd.recall_study (the Fig. 2 analogue): on a small stack its LRU hit ratio for k = top_k = 2
    equals the closed form sum_t |S_t & S_{t-1}| / needed, for k = E only the first touches miss; its speculative
    guesses -- taken by the library's gate kernel and top-m selection through moe_layer_prefetch -- give, for every
    (layers ahead, m) cell, exactly the integer counts of the oracle's definition (Sec. 4.1), and guessing all E
    experts recalls everything."""
    from paper_2312_17238_amd import recall_study as R
    shape = W.MoEShape("study", 5, 256, 512, 8, 2, 4, 64, 2, 2, 1e-5, 24, 1, "ar1", 5)
    routing, h_all, gates, stack = R.record(shape, W.layer_formats(shape), shape.tokens, "cuda:0")
    T, L = shape.tokens, shape.layers
    assert len(routing) == T and all(len(r) == L and all(len(s) == 2 for s in r) for r in routing)
    closed = sum(len(set(routing[t][l]) & set(routing[t - 1][l])) for t in range(1, T) for l in range(L)) / (2 * T * L)
    assert abs(R.lru_hit_ratio(routing, L, 8, 2, 2) - closed) < 1e-12
    touched = sum(len({e for t in range(T) for e in routing[t][l]}) for l in range(L))
    assert abs(R.lru_hit_ratio(routing, L, 8, 2, 8) - (1 - touched / (2 * T * L))) < 1e-12
    # the routing and the gate inputs the tool recorded are the oracle's
    gates_np, h_np = [g.numpy() for g in gates], h_all.numpy()
    for t in range(T):
        for l in range(L):
            idx, _, _ = O.route(gates_np[l], h_np[t, l], 2)
            assert list(idx) == routing[t][l]
    cells = {}
    for ahead in (1, 2, 4):
        guesses = R.speculative_guesses(stack, h_all, ahead)
        assert all(len(g) == 4 for row in guesses for g in row)
        for m in (1, 2, 4):
            got = R.speculative_recall_counts(routing, guesses, ahead, m)
            want = O.speculative_recall(routing, h_np, gates_np, ahead, m)
            assert got == want, f"{ahead} layers ahead, m={m}: library {got}, oracle {want}"
            cells[(ahead, m)] = got[0] / got[1]
        assert cells[(ahead, 1)] <= 0.5 and cells[(ahead, 1)] <= cells[(ahead, 2)] <= cells[(ahead, 4)] <= 1.0
    # all E experts guessed (the interface takes four guesses, so on a stack of four experts)
    stack.close()
    say(f"recall study: {cells}")
    small = W.MoEShape("study4", 3, 256, 512, 4, 2, 4, 64, 2, 2, 1e-5, 8, 1, "ar1", 6)
    routing, h_all, gates, stack = R.record(small, W.layer_formats(small), small.tokens, "cuda:0")
    got = R.speculative_recall_counts(routing, R.speculative_guesses(stack, h_all, 1), 1, 4)
    assert got == (2 * 8 * 2, 2 * 8 * 2) == O.speculative_recall(routing, h_all.numpy(), [g.numpy() for g in gates], 1, 4)
    stack.close()


@pytest.mark.parametrize("Bn,k,T,form", [(200, 4, 2, 3), (130, 2, 2, 1), (1000, 8, 1, 2), (1024, 2, 1, 3), (300, 4, 1, 2), (260, 4, 1, 4), (260, 4, 1, 5), (90, 2, 2, 5)])
def test_prompt_sized_batches(Bn, k, T, form):
    """Prompt encoding (Sec. 3: prompt tokens go through a layer in parallel, every expert is loaded once for all of
    them) is a step with a large batch: up to MOE_MAX_BATCH = 1024 tokens, through the matrix cores in windows of
    128 tokens per launch over the same resident experts; with k=2 and all 8 experts needed the step runs in
    several passes.  Every decision and every output row against the oracle."""
    L, H, F = 2, 256, 512
    say(f"prompt-sized batch B={Bn} k={k} form={form}")
    model = Model(L, H, F, 8, 2, None, k, 2, 1e-5, max_batch=Bn, seed=81)
    B.moe_ctx_set_option(model.stack.ctx, "mfma_form", form)
    B.moe_ctx_profile_enable(model.stack.ctx, True)
    xs = W.hidden_ar1(81, T, Bn, H)
    _, sim, errs = run_teacher_forced(model, xs, O.expert_ffn)
    prof = B.moe_ctx_profile_read(model.stack.ctx).as_dict()
    assert prof["w13"]["launches"] >= T * L * -(-Bn // 128)
    say(f"  max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e} w1/w3 launches {prof['w13']['launches']}")
    model.close()


@pytest.mark.parametrize("formats,scale_group,Bn", [([(2, 16), (3, 64)], 0, 300), ([(4, 64), (4, 64)], 256, 200)])
def test_prompt_sized_batches_on_the_gemv_kernels(formats, scale_group, Bn):
    """Formats the matrix-core kernels do not take (2-bit, 3-bit; and 4-bit with the threshold raised) run a large
    batch through the GEMV kernels, four tokens per entry and sixteen entries per launch."""
    L, H, F = 2, 256, 512
    say(f"prompt-sized batch on GEMV kernels B={Bn} formats={formats} scale_group={scale_group}")
    model = Model(L, H, F, 8, 2, formats, 4, 2, 1e-5, max_batch=Bn, seed=83, scale_group=scale_group)
    B.moe_ctx_set_option(model.stack.ctx, "mfma_min_batch", 100000)
    xs = W.hidden_ar1(83, 1, Bn, H)
    _, sim, errs = run_teacher_forced(model, xs, O.expert_ffn)
    say(f"  max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e}")
    model.close()


def draw_configuration(seed):
    """A seeded draw over shapes, formats, cache sizes, modes and launch options that the interface accepts."""
    r = np.random.RandomState(7000 + seed)
    pick = lambda xs: xs[int(r.randint(len(xs)))]
    c = {}
    c["E"] = pick([3, 4, 8, 8, 16])
    c["K"] = min(pick([1, 2, 2, 2, 3, 4]), c["E"])
    c["k"] = int(r.randint(c["K"], c["E"] + 1))
    c["m"] = pick([0, 1, 2, 2, 3, 4])
    c["L"] = pick([2, 3])
    c["H"] = pick([64, 192, 256, 320, 512, 768])       # any multiple of 64: ragged last chunks, blocks and tiles
    c["F"] = pick([64, 192, 320, 448, 512, 1024])
    c["Bn"] = pick([1, 1, 1, 2, 3, 5, 8, 16, 17, 40, 70])
    c["T"] = 6 if c["Bn"] <= 8 else 3
    c["formats"] = [pick([(4, 64), (4, 64), (3, 64), (2, 16)]) for _ in range(c["L"])]
    c["scale_group"] = pick([0, 0, 4, 8])
    c["swap"] = bool(r.rand() < 0.3)
    c["warm"] = c["swap"] or bool(r.rand() < 0.3)
    c["eps"] = pick([0.0, 1e-5])
    c["options"] = {
        "token_path": pick([1, 1, 0]), "fused": pick([0, 0, 0, 1, 2]), "mfma_form": pick([1, 2, 3, 4, 5, 0]), "mfma16_waves": pick([4, 8]),
        "mfma_min_batch": pick([16, 3, 2, 1000]), "staged_min_batch": pick([0, 0, 1000]),
        "spec_head_mb": pick([0, 0, 1]), "w13_blocks": pick([256, 64, 24]), "w2_rows": pick([32, 16, 8]),
        "sync_wait": pick([0, 0, 1]),
    }
    if r.rand() < 0.2:      # decode with every expert resident: the steps that do not wait for their gate
        c.update(Bn=1, T=6, k=c["E"], K=min(c["K"], 2))
        c["options"].update(token_path=1, fused=0)
    return c


def build_configuration(c, seed):
    model = Model(c["L"], c["H"], c["F"], c["E"], c["K"], c["formats"], c["k"], c["m"], c["eps"], max_batch=c["Bn"],
                  seed=7000 + seed, init_policy=1 if c["warm"] else 0, flags=B.MOE_LAYER_SWAP if c["swap"] else 0,
                  scale_group=c["scale_group"])
    for name, value in c["options"].items():
        B.moe_ctx_set_option(model.stack.ctx, name, value)
    return model


@pytest.mark.parametrize("seed", range(40))
def test_random_configurations(seed):
    """Forty seeded combinations of shapes, per-layer formats, metadata levels, cache sizes, swap mode, warm start
    and launch options, none of them chosen by hand: every decision bit-exact and every output row in tolerance
    against the oracle, as in the hand-picked cases above.  Then the same tokens through the whole-stack entry point
    without traces (after a reset, or on a stack built anew; statistics read at seeded moments, which makes
    device-routed steps catch up their bookkeeping there): the same counters and bit-identical outputs."""
    c = draw_configuration(seed)
    say(f"random configuration {seed}: {c}")
    model = build_configuration(c, seed)
    xs = W.hidden_ar1(7000 + seed, c["T"], c["Bn"], c["H"])
    sim = O.ExpertCacheSim(c["L"], c["E"], c["k"], 4, warm=c["warm"])
    place = [O.SwapPlacement(c["E"], c["k"]) for _ in range(c["L"])] if c["swap"] else None
    outs, sim, errs = run_teacher_forced(model, xs, O.expert_ffn, sim=sim, placement=place)
    tot = model.stack.total_stats()
    assert tot["needed"] == sum(s.needed for s in sim.stats)
    assert tot["misses"] == sum(s.misses for s in sim.stats)
    assert tot["prefetch_hits"] == sum(s.prefetch_hits for s in sim.stats)
    say(f"  max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e} misses {tot['misses']}")
    r = np.random.RandomState(9000 + seed)
    if c["swap"] or r.rand() < 0.5:          # a layer in swap mode cannot be reset
        model.close()
        model = build_configuration(c, seed)
    else:
        model.stack.reset()
    dev = model.stack.device
    x_in = torch.empty(c["Bn"], c["H"], dtype=torch.float16, device=dev)
    x_out = torch.empty(c["Bn"], c["H"], dtype=torch.float16, device=dev)
    # no kernel of the path adds with atomics: a pair's output has one writer and a token's pairs (and the parts of a
    # contraction split over blocks) are added in a fixed order, so the free-running pass must reproduce the
    # teacher-forced one -- which was checked against the oracle above -- bit for bit, with the same counters
    for t in range(c["T"]):
        x_in.copy_(xs[t])
        torch.cuda.synchronize()
        model.stack.step(x_in, x_out, None)
        if r.rand() < 0.4:
            model.stack.total_stats()
        model.stack.synchronize()
        got = x_out.cpu().numpy()
        differ = got.view(np.uint16) != outs[t].view(np.uint16)
        gap = np.abs(got.astype(np.float64) - outs[t].astype(np.float64))
        assert not differ.any(), f"whole-stack step differs at token {t}: {int(differ.sum())} of {differ.size} elements, largest gap {gap.max():.3e}"
    again = model.stack.total_stats()
    for name in ("needed", "hits", "misses", "prefetch_hits", "evictions", "spec_issued", "spec_wasted", "bytes_d2h_writeback"):
        assert again[name] == tot[name], f"{name}: {again[name]} after the whole-stack pass, {tot[name]} before"
    say(f"  whole-stack pass: device-routed steps {again['steps_device_routed']}")
    model.close()


@pytest.mark.parametrize("factor,falls_back", [(1, False), (8192, True)])
def test_rank1_matrix_core_form_gives_way_to_large_scales(factor, falls_back):
    """The default matrix-core form forms (1024 + zero) * scale in fp16.  A layer that was loaded with a (scale, zero)
    pair for which that product leaves the comfortable part of the fp16 range runs the form that subtracts first
    instead: asking for form 3 then gives bit for bit what asking for form 2 gives (two addends per element here, so
    the sums do not depend on their order), while on ordinary weights the two forms differ in the last bits.  The
    group-scaled form 5 works in fp32 and takes any pair: it stays in tolerance of form 2 either way."""
    H, F, Bn = 256, 512, 16
    say(f"rank-1 form and scales x{factor}")
    model = Model(1, H, F, 8, 2, None, 8, 0, 0.0, max_batch=Bn, seed=77, keep_layers=[])
    for e in range(8):
        for mtx, (codes, scale, zero) in enumerate(W.quantized_expert(77, 0, e, H, F, 4, 64, model.device, 0)):
            model.stack.load_expert(0, e, mtx, codes, (scale.float() * factor).half(), zero)
    dev = model.stack.device
    x_in = (W.hidden_ar1(77, 1, Bn, H)[0].float() / factor).half().to(dev)      # keeps the outputs in range
    x_out = torch.empty(Bn, H, dtype=torch.float16, device=dev)
    ys = {}
    for form in (3, 2, 5):
        B.moe_ctx_set_option(model.stack.ctx, "mfma_form", form)
        model.stack.step_layer(0, x_in, x_out, None, None, prefetch=False)
        model.stack.synchronize()
        ys[form] = model.stack.read_y(Bn, H).copy()
        assert np.isfinite(ys[form]).all() and np.abs(ys[form]).max() > 0
    same = (ys[3].view(np.uint32) == ys[2].view(np.uint32)).all()
    assert same == falls_back, f"forms 3 and 2 {'agree' if same else 'differ'} bit for bit"
    d = np.abs(ys[5] - ys[2]).max()
    assert d <= 2e-3 * np.abs(ys[2]).max(), f"form 5 against form 2: {d:.3e} of {np.abs(ys[2]).max():.3e}"
    model.close()


@pytest.mark.parametrize("E,K,k,Bn,path", [(8, 4, 8, 16, "matrix"), (8, 2, 8, 20, "matrix"), (16, 4, 4, 64, "matrix"), (8, 4, 4, 6, "gemv"),
                                           (8, 3, 8, 1, "gemv")])
def test_block_output_is_reproducible_bit_for_bit(E, K, k, Bn, path):
    """y has up to four addends per element (top-k above 2) and, on the matrix cores, a contraction split over
    blocks whose partial sums arrive in any order.  None of them is added with atomics: the same step on two stacks
    built alike, and again on the first, gives the same fp32 y to the last bit (and an in-tolerance one)."""
    L, H, F = 1, 256, 1024
    xs = W.hidden_ar1(131, 3, Bn, H)
    ys = []
    models = [Model(L, H, F, E, K, None, k, 0, 1e-5, max_batch=Bn, seed=131) for _ in range(2)]
    for model in models:
        B.moe_ctx_set_option(model.stack.ctx, "mfma_min_batch", 16 if path == "matrix" else 1000)
    dev = models[0].stack.device
    for rep, model in enumerate((models[0], models[1], models[0])):
        if rep == 2:
            model.stack.reset()
        x_out = torch.empty(Bn, H, dtype=torch.float16, device=dev)
        row = []
        for t in range(xs.shape[0]):
            x_in = xs[t].to(dev)
            tr = B.StepTrace()
            model.stack.step_layer(0, x_in, x_out, None, tr)
            model.stack.synchronize()
            y = model.stack.read_y(Bn, H).copy()
            if rep == 0:
                for bb, (h, idx, w, _) in enumerate(oracle_routing(model, 0, xs[t].numpy())):
                    assert tr.routing()[bb] == idx
                    check_y(y[bb], oracle_y(model, 0, h, idx, w, O.expert_ffn), f"y t={t} b={bb}")
            row.append((y, x_out.cpu().numpy().copy()))
        ys.append(row)
    for other in ys[1:]:
        for (ya, xa), (yb, xb) in zip(ys[0], other):
            assert (ya.view(np.uint32) == yb.view(np.uint32)).all() and (xa.view(np.uint16) == xb.view(np.uint16)).all()
    for model in models:
        model.close()


@pytest.mark.parametrize("H,F,k,Bn,path", [(256, 1024, 4, 16, "matrix"), (256, 1024, 8, 48, "matrix"), (1024, 2048, 4, 16, "matrix"),
                                           (256, 1024, 4, 6, "gemv"), (256, 1024, 2, 1, "gemv")])
def test_block_output_does_not_depend_on_what_the_cache_held(H, F, k, Bn, path):
    """Sec. 3.2: caching and speculative loading change no prediction.  Here that holds to the last bit: the same
    tokens give the same fp32 y from a cold cache (every expert arrives during the step, one launch per arrival or
    several passes), from a warm one (resident experts first, in one launch), after a reset (the experts land in
    other buffers, which groups the launches differently) and with speculative loading on or off."""
    L, E, K = 2, 8, 2
    xs = W.hidden_ar1(137, 2, Bn, H)
    model = Model(L, H, F, E, K, None, k, 2, 1e-5, max_batch=Bn, seed=137, keep_layers=[])
    B.moe_ctx_set_option(model.stack.ctx, "mfma_min_batch", 16 if path == "matrix" else 1000)
    dev = model.stack.device
    x_in = [xs[t].to(dev) for t in range(2)]
    def run():
        ys = []
        for t in (0, 1, 0, 1):                      # the second visit of a token finds the cache warm
            xa, xb2 = torch.empty(Bn, H, dtype=torch.float16, device=dev), torch.empty(Bn, H, dtype=torch.float16, device=dev)
            model.stack.step_layer(0, x_in[t], xa, None, B.StepTrace())
            model.stack.synchronize()
            y0 = model.stack.read_y(Bn, H).copy()
            model.stack.step_layer(1, xa, xb2, None, None)
            model.stack.synchronize()
            ys.append((y0, model.stack.read_y(Bn, H).copy()))
        return ys
    first = run()
    for a, b in ((0, 2), (1, 3)):
        for l in range(2):
            assert (first[a][l].view(np.uint32) == first[b][l].view(np.uint32)).all(), f"cold and warm differ, token {a} layer {l}"
    model.stack.reset()
    again = run()
    model.stack.reset()
    model.stack.set_prefetch(0)
    without = run()
    for other, what in ((again, "after a reset"), (without, "without speculative loading")):
        for i in range(4):
            for l in range(2):
                assert (first[i][l].view(np.uint32) == other[i][l].view(np.uint32)).all(), f"{what}: visit {i} layer {l} differs"
    model.close()


@pytest.mark.parametrize("fused", [2, 1])
def test_mixtral_layer_one_launch_kernels(fused):
    """The single-token FFN as ONE persistent launch at Mixtral size, where 256 blocks on eight dies hand the
    activations a to each other through memory inside the kernel (2: expert after expert, flags per expert; 1: one
    grid barrier): k=2, so nearly every step also waits for 99 MB copies; C oracle on every token, and outputs
    bit-identical to the two-launch path."""
    c = W.CONFIGS["mixtral_layer"]
    xs = W.hidden_ar1(c.seed + 1, 10, 1, c.hidden)
    res = {}
    for mode in (fused, 0):
        say(f"mixtral layer, fused={mode}: build")
        model = Model(1, c.hidden, c.ffn, c.n_experts, c.top_k, None, 2, 0, 0.0, seed=c.seed, keep_layers=[] if mode == 0 else None)
        B.moe_ctx_set_option(model.stack.ctx, "fused", mode)
        B.moe_ctx_profile_enable(model.stack.ctx, True)
        outs, sim, errs = run_teacher_forced(model, xs, c_ffn.expert_ffn, check_ffn=lambda t, l: mode != 0)
        prof = B.moe_ctx_profile_read(model.stack.ctx).as_dict()
        assert (prof["ffn"]["launches"] == 10) == (mode != 0) and (prof["w13"]["launches"] == 10) == (mode == 0)
        if errs:
            say(f"  max abs {max(e[0] for e in errs):.2e} max rel-rms {max(e[1] for e in errs):.2e}")
        res[mode] = outs
        model.close()
    for a, b in zip(res[fused], res[0]):
        assert (a.view(np.uint16) == b.view(np.uint16)).all()

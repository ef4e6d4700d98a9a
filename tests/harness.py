"""Shared test plumbing: build an engine Stack from a synthetic workload and keep what the oracle
needs (unpacked codes, scales, zeros as numpy) on the host.  No arithmetic of the method lives here."""
from __future__ import annotations

import sys
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

import workload as W
from oracle import moe_oracle as O
from paper_2312_17238_amd import binding as B
from paper_2312_17238_amd.engine import Stack, layer_config

TOL_MAX_ABS = 2e-2      # the benchmark definition's bound on fp16 FFN outputs
TOL_REL_RMS = 1e-3


def to_np_expert(mats):
    return [tuple(t.cpu().numpy() if hasattr(t, "cpu") else t for t in m) for m in mats]


class Model:
    """L layers of E experts each: the engine Stack plus the host copies the oracle reads."""

    def __init__(self, L, H, F, E=8, K=2, formats: Optional[Sequence[Tuple[int, int]]] = None, k=2, m=0,
                 rms_eps=0.0, b=4, max_batch=1, seed=0, device="cuda:0", keep_layers: Optional[Sequence[int]] = None,
                 init_policy=0, flags=0, scale_group=0):
        self.L, self.H, self.F, self.E, self.K, self.k, self.m, self.eps = L, H, F, E, K, k, m, rms_eps
        self.formats = list(formats) if formats else [(4, 64)] * L
        self.scale_group = scale_group      # > 0: two-level metadata (8-bit scale and zero codes, fp16 quads per run)
        self.seed = seed
        self.device = device
        self.memo = None
        self.gate = [W.gate_weight(seed, l, E, H) for l in range(L)]
        self.gamma = [W.rms_gamma(H) for _ in range(L)] if rms_eps > 0 else None
        cfgs = [layer_config(H, F, E, K, self.formats[l][0], self.formats[l][1], k, m, rms_eps, init_policy, flags,
                             scale_group) for l in range(L)]
        self.stack = Stack(cfgs, self.gate, self.gamma, n_staging=b, max_batch=max_batch, device=device)
        self.experts: Dict[Tuple[int, int], list] = {}
        keep = set(range(L)) if keep_layers is None else set(keep_layers)
        for l in range(L):
            bits, group = self.formats[l]
            for e in range(E):
                mats = W.quantized_expert(seed, l, e, H, F, bits, group, device, scale_group)
                for mtx, m in enumerate(mats):
                    self.stack.load_expert(l, e, mtx, *m)
                if l in keep:
                    self.experts[(l, e)] = to_np_expert(mats)
                del mats

    def expert_np(self, l, e):
        """Unpacked (codes, scale, zero) of one expert; regenerated from its seed if not kept (and remembered while
        `memo` is a dict: the rows of one step that are checked against the oracle share their experts)."""
        if (l, e) in self.experts:
            return self.experts[(l, e)]
        if self.memo is not None and (l, e) in self.memo:
            return self.memo[(l, e)]
        bits, group = self.formats[l]
        ex = to_np_expert(W.quantized_expert(self.seed, l, e, self.H, self.F, bits, group, self.device, self.scale_group))
        if self.memo is not None:
            self.memo[(l, e)] = ex
        return ex

    def gate_np(self, l):
        return self.gate[l].numpy()

    def gamma_np(self, l):
        return self.gamma[l].numpy() if self.gamma is not None else None

    def close(self):
        self.stack.close()


def oracle_routing(model: Model, l: int, x_f16: np.ndarray):
    """Per token: gate input h, selection, weights, logits -- from the oracle, for the x the engine consumed."""
    out = []
    for b in range(x_f16.shape[0]):
        h = O.rmsnorm(x_f16[b], model.gamma_np(l), model.eps) if model.eps > 0 else x_f16[b]
        idx, w, z = O.route(model.gate_np(l), h, model.K)
        out.append((h, idx, w, z))
    return out


def oracle_y(model: Model, l: int, h: np.ndarray, idx, w, ffn) -> np.ndarray:
    y = np.zeros(model.H, dtype=np.float64)
    for j, e in enumerate(idx):
        y = y + w[j] * ffn(h, model.expert_np(l, e), model.formats[l][1])
    return y


def check_y(y_gpu: np.ndarray, y_ref: np.ndarray, what: str):
    err = np.abs(y_gpu.astype(np.float64) - y_ref)
    rel = float(np.linalg.norm(y_gpu.astype(np.float64) - y_ref) / max(np.linalg.norm(y_ref), 1e-30))
    assert err.max() <= TOL_MAX_ABS, f"{what}: max abs error {err.max():.3e} > {TOL_MAX_ABS}"
    assert rel <= TOL_REL_RMS, f"{what}: relative RMS error {rel:.3e} > {TOL_REL_RMS}"
    return float(err.max()), rel


def check_x_out(x_out_gpu: np.ndarray, x_f16: np.ndarray, y_ref: np.ndarray, what: str):
    want = x_f16.astype(np.float64) + y_ref
    err = np.abs(x_out_gpu.astype(np.float64) - want)
    # fp16 rounding of the sum (half an ulp of the result) on top of the FFN tolerance
    ulp = np.maximum(np.abs(want), 2.0 ** -14) * 2.0 ** -10
    assert (err <= TOL_MAX_ABS + ulp).all(), f"{what}: x_out off by {err.max():.3e}"


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def run_teacher_forced(model: Model, xs: torch.Tensor, ffn, check_ffn=lambda t, l: True, prefetch=True, b=4,
                       sim=None, placement=None, rows=None):
    """xs: [T][B][H] fp16 (CPU).  Runs layer by layer, checks every decision, returns (final x per token, sim, errs).
    placement: per layer an oracle SwapPlacement to follow and compare with the engine's after every step.
    check_ffn(t, l): compare the block output of that step with the oracle -- every batch row, or those rows(t, l) names."""
    L, E, K = model.L, model.E, model.K
    T, Bn, H = xs.shape
    sim = sim or O.ExpertCacheSim(L, E, model.k, b)
    dev = model.stack.device
    xb = [torch.empty(Bn, H, dtype=torch.float16, device=dev) for _ in range(L + 1)]
    hb = torch.empty(Bn, H, dtype=torch.float16, device=dev)
    outs, errs = [], []
    for t in range(T):
        xb[0].copy_(xs[t])
        torch.cuda.synchronize()
        for l in range(L):
            tr = B.StepTrace()
            model.stack.step_layer(l, xb[l], xb[l + 1], hb, tr, prefetch=prefetch)
            model.stack.synchronize()
            x_np = xb[l].cpu().numpy()
            routes = oracle_routing(model, l, x_np)
            h_ref = np.stack([r[0] for r in routes])
            assert (hb.cpu().numpy().view(np.uint16) == h_ref.view(np.uint16)).all(), f"gate input differs t={t} l={l}"
            sel = [r[1] for r in routes]
            assert tr.routing() == sel, f"routing differs t={t} l={l}: {tr.routing()} vs {sel}"
            w_ref = np.array([r[2] for r in routes])
            assert np.abs(np.array(tr.weights()) - w_ref).max() < 1e-6
            z_ref = np.array([r[3] for r in routes])
            z_gpu = np.array(tr.logits[: Bn * E]).reshape(Bn, E)
            assert np.abs(z_gpu - z_ref).max() <= 1e-12 * max(1.0, np.abs(z_ref).max())
            guess = None
            if prefetch and l + 1 < L and model.m > 0:
                guess = O.prefetch_guess(O.prefetch_scores(model.gate_np(l + 1), h_ref), model.m)
            acc, dec = sim.step(l, sel, guess)
            assert tr.accesses() == [(a.expert, a.status, a.slot, a.victim) for a in acc], f"cache trace differs t={t} l={l}"
            assert tr.guesses() == [(e, i) for e, i in dec], f"prefetch decisions differ t={t} l={l}"
            if placement is not None:
                placement[l].apply(acc)
                assert B.moe_layer_placement(model.stack.layers[l], E) == (placement[l].host_buf_of, placement[l].spare), \
                    f"placement differs t={t} l={l}"
            if check_ffn(t, l):
                y_gpu = model.stack.read_y(Bn, H)
                x_out = xb[l + 1].cpu().numpy()
                model.memo = {}
                for bb in (range(Bn) if rows is None else rows(t, l)):
                    h, idx, w, _ = routes[bb]
                    y_ref = oracle_y(model, l, h, idx, w, ffn)
                    errs.append(check_y(y_gpu[bb], y_ref, f"y t={t} l={l} b={bb}"))
                    check_x_out(x_out[bb], x_np[bb], y_ref, f"x_out t={t} l={l} b={bb}")
                model.memo = None
        outs.append(xb[L].cpu().numpy().copy())
    return outs, sim, errs

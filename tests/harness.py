"""Shared test plumbing: build an engine Stack from a synthetic workload and keep what the oracle
needs (unpacked codes, scales, zeros as numpy) on the host.  No arithmetic of the method lives here."""
from __future__ import annotations

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
        """Unpacked (codes, scale, zero) of one expert; regenerated from its seed if not kept."""
        if (l, e) not in self.experts:
            bits, group = self.formats[l]
            return to_np_expert(W.quantized_expert(self.seed, l, e, self.H, self.F, bits, group, self.device, self.scale_group))
        return self.experts[(l, e)]

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

"""Memory plumbing around the C ABI: PyTorch allocates the device arenas, the pinned host arenas
and the two streams; every computation happens inside libmoe_offload.so."""
from __future__ import annotations

import ctypes as C
from typing import List, Optional, Sequence

import numpy as np
import torch

from . import binding as B


def layer_config(hidden, ffn, n_experts=8, top_k=2, bits=4, group=64, cache_slots=2, prefetch_m=0,
                 rms_eps=0.0, init_policy=0, flags=0, scale_group=0) -> B.LayerConfig:
    return B.LayerConfig(hidden, ffn, n_experts, top_k, bits, group, cache_slots, prefetch_m, rms_eps,
                         init_policy, flags, scale_group)


class Stack:
    """A context plus L layers.  `host_only=True` builds the bookkeeping-only variant (no GPU)."""

    def __init__(self, cfgs: Sequence[B.LayerConfig], gate_w: Sequence[torch.Tensor],
                 gamma: Optional[Sequence[Optional[torch.Tensor]]] = None, n_staging: int = 4,
                 max_batch: int = 1, device: str = "cuda:0", host_only: bool = False):
        self.cfgs = list(cfgs)
        self.L = len(self.cfgs)
        self.host_only = host_only
        self.device = torch.device(device) if not host_only else torch.device("cpu")
        self.max_batch = max_batch
        blob = [B.moe_expert_blob_bytes(c.hidden, c.ffn, c.bits, c.group, c.scale_group) for c in self.cfgs]
        if min(blob) == 0:
            raise B.MoeError(B.MOE_EINVAL, "unsupported shape or format")
        self.blob_bytes = blob
        cc = B.CtxConfig(n_staging, max_batch, max(c.hidden for c in self.cfgs), max(c.ffn for c in self.cfgs),
                         max(c.top_k for c in self.cfgs), B.MOE_CTX_HOST_ONLY if host_only else 0, max(blob))
        self.ctx_cfg = cc
        self._keep = []
        if host_only:
            self.ctx = B.moe_ctx_create(cc, None, 0, None, None)
        else:
            torch.cuda.set_device(self.device)
            self.compute = torch.cuda.Stream(device=self.device)
            self.copy = torch.cuda.Stream(device=self.device)
            n = B.moe_ctx_dev_bytes(cc)
            self.arena = torch.empty(n, dtype=torch.uint8, device=self.device)
            self.ctx = B.moe_ctx_create(cc, self.arena.data_ptr(), n, self.compute.cuda_stream, self.copy.cuda_stream)
        self.layers = []
        self.host_arenas = []
        self.dev_mems = []
        for l, c in enumerate(self.cfgs):
            hb = B.moe_layer_host_bytes(c)
            if host_only:
                host = torch.empty(hb, dtype=torch.uint8)
                dev_ptr = None
            else:
                host = torch.empty(hb, dtype=torch.uint8, pin_memory=True)
                dm = torch.empty(B.moe_layer_dev_bytes(self.ctx, c), dtype=torch.uint8, device=self.device)
                self.dev_mems.append(dm)
                dev_ptr = dm.data_ptr()
            self.host_arenas.append(host)
            gw = gate_w[l].detach().to("cpu", torch.float32).contiguous()
            g = None
            if gamma is not None and gamma[l] is not None:
                g = gamma[l].detach().to("cpu", torch.float16).contiguous()
            self._keep += [gw, g]
            self.layers.append(B.moe_layer_create(self.ctx, c, gw.data_ptr(), g.data_ptr() if g is not None else None,
                                                  dev_ptr, host.data_ptr()))
        self._stage = {}

    # -- loading -----------------------------------------------------------------------------
    def _host(self, t: torch.Tensor, key: str) -> torch.Tensor:
        """A contiguous host copy of `t` (through a reusable pinned staging tensor if it is on the GPU)."""
        if t.device.type == "cpu":
            return t.contiguous()
        buf = self._stage.get(key)
        if buf is None or buf.numel() < t.numel() or buf.dtype != t.dtype:
            buf = torch.empty(t.numel(), dtype=t.dtype, pin_memory=True)
            self._stage[key] = buf
        view = buf[: t.numel()].view(t.shape)
        view.copy_(t, non_blocking=False)
        return view

    def load_expert(self, layer: int, expert: int, matrix: int, codes: torch.Tensor, scale: torch.Tensor,
                    zero: torch.Tensor, run_meta: Optional[torch.Tensor] = None, run_len: Optional[int] = None) -> None:
        """One-level metadata: scale, zero fp16 per group.  Two-level (run_meta given): scale, zero are the byte
        codes per group and run_meta the fp16 quads [out][runs][4]; run_len, if given, is checked against the
        groups per run the layer was configured with."""
        c = self._host(codes, "c")
        s = self._host(scale, "s")
        z = self._host(zero, "z")
        if run_meta is None:
            assert c.dtype == torch.uint8 and s.dtype == torch.float16 and z.dtype == torch.float16
            B.moe_layer_load_expert(self.layers[layer], expert, matrix, c.data_ptr(), s.data_ptr(), z.data_ptr())
        else:
            m = self._host(run_meta, "m")
            if run_len is not None and run_len != min(self.cfgs[layer].scale_group, s.shape[1]):
                raise ValueError(f"expert quantized with runs of {run_len} groups, layer configured for {self.cfgs[layer].scale_group}")
            assert c.dtype == torch.uint8 and s.dtype == torch.uint8 and z.dtype == torch.uint8 and m.dtype == torch.float16
            B.moe_layer_load_expert_2level(self.layers[layer], expert, matrix, c.data_ptr(), s.data_ptr(), z.data_ptr(),
                                           m.data_ptr())

    # -- stepping ----------------------------------------------------------------------------
    def step_layer(self, layer: int, x_in: torch.Tensor, x_out: torch.Tensor, h_out: Optional[torch.Tensor] = None,
                   trace: Optional[B.StepTrace] = None, prefetch: bool = True) -> None:
        nxt = self.layers[layer + 1] if (prefetch and layer + 1 < self.L) else None
        B.moe_layer_step(self.layers[layer], nxt, x_in.data_ptr(), x_in.shape[0], x_out.data_ptr(),
                         h_out.data_ptr() if h_out is not None else None, trace)

    def step(self, x_in: torch.Tensor, x_out: torch.Tensor, traces=None) -> None:
        B.moe_stack_step(self.layers, x_in.data_ptr(), x_in.shape[0], x_out.data_ptr(), traces)

    def read_y(self, batch: int, hidden: int) -> np.ndarray:
        y = np.empty((batch, hidden), dtype=np.float32)
        B.moe_ctx_read_y(self.ctx, batch, hidden, y.ctypes.data)
        return y

    def synchronize(self) -> None:
        if not self.host_only:
            self.compute.synchronize()
            self.copy.synchronize()

    # -- state -------------------------------------------------------------------------------
    def stats(self) -> List[dict]:
        return [B.moe_layer_stats(l).as_dict() for l in self.layers]

    def total_stats(self) -> dict:
        tot = {}
        for s in self.stats():
            for k, v in s.items():
                tot[k] = tot.get(k, 0) + v
        return tot

    def reset(self) -> None:
        for l in self.layers:
            B.moe_layer_reset(l)

    def set_prefetch(self, m: int) -> None:
        for l in self.layers:
            B.moe_layer_set_prefetch(l, m)

    def set_flags(self, flags: int) -> None:
        for l in self.layers:
            B.moe_layer_set_flags(l, flags)

    def close(self) -> None:
        if getattr(self, "layers", None):
            self.synchronize()
            for l in self.layers:
                B.moe_layer_destroy(l)
            self.layers = []
        if getattr(self, "ctx", None):
            B.moe_ctx_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def make_traces(n: int):
    return (B.StepTrace * n)()

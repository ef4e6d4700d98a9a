"""Seeded synthetic inputs with the shapes and value structure of the paper's workload.

The paper (Sec. 4.3) measures Mixtral-8x7B-Instruct on OpenAssistant prompts;
neither is available offline, so every input here is synthetic:

* gate matrices  W_g ~ N(0, 0.02) in fp32, one [E, H] matrix per layer;
* expert matrices ~ N(0, 0.02) in fp32, quantized group-wise with a plain
  asymmetric min/max quantizer to 2/3/4-bit codes plus fp16 scale and zero
  per group (the formats of Sec. 4.2, with fp16 metadata);
* hidden states: i.i.d. N(0,1) per token (tiny config) or an AR(1) stream
  x_t = rho x_{t-1} + eps_t with rho = 0.8 so that adjacent tokens reuse
  experts, the regularity Sec. 3.1 builds the LRU cache on.

All streams derive from one integer seed through `stream_seed`, keyed by
(kind, layer, expert, matrix, stream), so any single tensor can be regenerated
without generating the others.  Small tensors (gates, hidden states) are always
drawn on the CPU so they are identical on every machine; expert matrices are
drawn on the requested device (torch's Philox streams differ between CPU and
GPU, each deterministic for its device type).
"""
from __future__ import annotations

import dataclasses
import hashlib
from typing import Dict, List, Tuple

import torch

KIND_GATE = 1
KIND_EXPERT = 2
KIND_HIDDEN = 3
KIND_FORMAT = 4

W1, W3, W2 = 0, 1, 2  # matrix ids: w1 [F,H], w3 [F,H], w2 [H,F]


@dataclasses.dataclass(frozen=True)
class MoEShape:
    name: str
    layers: int
    hidden: int
    ffn: int
    n_experts: int
    top_k: int
    bits: int          # 0 => mixed per layer (see layer_formats)
    group: int
    cache_slots: int
    prefetch_m: int
    rms_eps: float     # 0 => no RMSNorm, no residual stack semantics beyond x+y
    tokens: int
    batch: int
    hidden_kind: str   # "iid" | "ar1"
    seed: int = 0


CONFIGS: Dict[str, MoEShape] = {
    # tiny single layer, every token checked against the oracle
    "tiny": MoEShape("tiny", 1, 256, 512, 8, 2, 4, 64, 2, 0, 0.0, 64, 1, "iid"),
    # one Mixtral-shaped layer, all experts resident: the pure dequant-GEMV measurement
    "mixtral_layer": MoEShape("mixtral_layer", 1, 4096, 14336, 8, 2, 4, 64, 8, 0, 0.0, 256, 1, "ar1"),
    # the headline: 32-layer stack, 4-bit, k=2, speculative prefetch of 2
    "mixtral_stack": MoEShape("mixtral_stack", 32, 4096, 14336, 8, 2, 4, 64, 2, 2, 1e-5, 512, 1, "ar1"),
    # mixed 2-bit g16 / 3-bit g64 per layer, k=4
    "mixtral_stack_lowbit": MoEShape("mixtral_stack_lowbit", 32, 4096, 14336, 8, 2, 0, 0, 4, 2, 1e-5, 512, 1, "ar1"),
    # batched decode, k=4 (batch is swept by the caller: 1, 4, 16, 64)
    "mixtral_stack_batched": MoEShape("mixtral_stack_batched", 32, 4096, 14336, 8, 2, 4, 64, 4, 2, 1e-5, 128, 64, "ar1"),
}


def stream_seed(seed: int, kind: int, layer: int = 0, expert: int = 0, matrix: int = 0, stream: int = 0) -> int:
    """63-bit sub-stream seed from the master seed and the tensor's coordinates."""
    key = f"{seed}:{kind}:{layer}:{expert}:{matrix}:{stream}".encode()
    return int.from_bytes(hashlib.blake2b(key, digest_size=8).digest(), "little") & ((1 << 63) - 1)


def _gen(device, s: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(s)
    return g


def gate_weight(seed: int, layer: int, n_experts: int, hidden: int) -> torch.Tensor:
    """fp32 [E, H] ~ N(0, 0.02), drawn on the CPU."""
    g = _gen("cpu", stream_seed(seed, KIND_GATE, layer))
    return torch.randn(n_experts, hidden, generator=g, dtype=torch.float32) * 0.02


def rms_gamma(hidden: int) -> torch.Tensor:
    """RMSNorm gain: ones, fp16."""
    return torch.ones(hidden, dtype=torch.float16)


def expert_matrix_shape(matrix: int, hidden: int, ffn: int) -> Tuple[int, int]:
    """[out, in] of w1/w3 (hidden -> ffn) and w2 (ffn -> hidden)."""
    return (ffn, hidden) if matrix in (W1, W3) else (hidden, ffn)


def expert_matrix(seed: int, layer: int, expert: int, matrix: int, hidden: int, ffn: int,
                  device="cpu") -> torch.Tensor:
    """fp32 [out, in] ~ N(0, 0.02) on `device`."""
    out_f, in_f = expert_matrix_shape(matrix, hidden, ffn)
    g = _gen(device, stream_seed(seed, KIND_EXPERT, layer, expert, matrix))
    return torch.randn(out_f, in_f, generator=g, dtype=torch.float32, device=device) * 0.02


META8_ZERO_LIMIT = 60000.0   # largest |zero| a run's fp16 pair may carry (fp16 overflows at 65520)


def quantize_minmax(w: torch.Tensor, bits: int, group: int, zero_limit=None):
    """Asymmetric min/max group quantization along the input (last) dimension.

    Per group of `group` consecutive elements of a row: lo = min, hi = max,
    scale = fp16((hi - lo) / (2^bits - 1)) (1 if that rounds to 0),
    zero = fp16(-lo / scale) (real-valued, not rounded to an integer),
    code = clamp(rint(w / scale + zero), 0, 2^bits - 1), using the rounded fp16
    scale and zero, all arithmetic in fp32.

    Returns (codes uint8 [out, in], scale fp16 [out, in/group], zero fp16 [out, in/group]).

    zero_limit (second level only): a group whose |lo / scale| would exceed it (values close together
    relative to their size; the zero would overflow fp16) is stored as a constant: scale = 1,
    zero = fp16(-lo), all codes 0.
    """
    out_f, in_f = w.shape
    assert in_f % group == 0
    qmax = float((1 << bits) - 1)
    wg = w.reshape(out_f, in_f // group, group).to(torch.float32)
    lo = wg.amin(dim=2)
    hi = wg.amax(dim=2)
    s16 = ((hi - lo) / qmax).to(torch.float16)
    s16 = torch.where(s16 == 0, torch.ones_like(s16), s16)
    if zero_limit is not None:
        s16 = torch.where((lo / s16.to(torch.float32)).abs() > zero_limit, torch.ones_like(s16), s16)
    sf = s16.to(torch.float32)
    z16 = (-lo / sf).to(torch.float16)
    zf = z16.to(torch.float32)
    q = torch.round(wg / sf.unsqueeze(2) + zf.unsqueeze(2)).clamp_(0.0, qmax)
    return q.to(torch.uint8).reshape(out_f, in_f), s16, z16


def run_length(groups: int, scale_group: int) -> int:
    """Groups per run of the second quantization level: scale_group, or the whole row if it has fewer groups.
    A row whose groups do not divide into whole runs ends in a shorter one."""
    return min(scale_group, groups)


def quantize_meta8(scale_f16: torch.Tensor, zero_f16: torch.Tensor, scale_group: int):
    """Second quantization level (Sec. 4.2 "scale group size"): the fp16 scales, and separately the fp16 zeros,
    of a row are themselves quantized to 8 bits with the same min/max rule, in runs of `scale_group`
    consecutive groups of that row (the whole row if it has fewer), each run with an fp16 (scale, zero) of its own.

    Returns (scale codes u8 [out, in/g], zero codes u8 [out, in/g], meta fp16 [out, runs, 4], groups per run) with
    meta[r, j] = (scale of the scale codes, zero of the scale codes, scale of the zero codes, zero of the zero codes).
    """
    groups = scale_f16.shape[1]
    r = run_length(groups, scale_group)
    runs = (groups + r - 1) // r

    def level2(v16):
        v = v16.to(torch.float32)
        if runs * r > groups:      # short last run: repeat its last value, which leaves its minimum and maximum alone
            v = torch.cat([v, v[:, -1:].expand(-1, runs * r - groups)], dim=1)
        q, s, z = quantize_minmax(v, 8, r, META8_ZERO_LIMIT)
        return q[:, :groups].contiguous(), s, z

    qs, ss, sz = level2(scale_f16)
    qz, zs, zz = level2(zero_f16)
    return qs, qz, torch.stack([ss, sz, zs, zz], dim=2).contiguous(), r


def quantized_expert(seed: int, layer: int, expert: int, hidden: int, ffn: int, bits: int, group: int,
                     device="cpu", scale_group: int = 0):
    """[(codes, scale, zero)] for matrices w1, w3, w2 of one expert; with scale_group > 0
    [(codes, scale codes, zero codes, meta, groups per run)] (see quantize_meta8)."""
    out = []
    for m in (W1, W3, W2):
        w = expert_matrix(seed, layer, expert, m, hidden, ffn, device)
        q, s, z = quantize_minmax(w, bits, group)
        out.append((q,) + quantize_meta8(s, z, scale_group) if scale_group else (q, s, z))
        del w
    return out


def hidden_iid(seed: int, tokens: int, batch: int, hidden: int) -> torch.Tensor:
    """fp16 [tokens, batch, hidden], i.i.d. N(0,1), drawn on the CPU."""
    g = _gen("cpu", stream_seed(seed, KIND_HIDDEN, 0, 0, 0, 0))
    return torch.randn(tokens, batch, hidden, generator=g, dtype=torch.float32).to(torch.float16)


def hidden_ar1(seed: int, tokens: int, batch: int, hidden: int, rho: float = 0.8) -> torch.Tensor:
    """fp16 [tokens, batch, hidden]: independent AR(1) streams per batch row.

    x_0 ~ N(0, 1/(1-rho^2)) (the stationary law), x_t = rho x_{t-1} + eps_t with
    eps ~ N(0,1) i.i.d. per element; the state is kept in fp32 and cast to fp16
    per token.  Batch row b uses sub-stream b, so a batch-B run sees the same
    first rows as a batch-1 run.
    """
    out = torch.empty(tokens, batch, hidden, dtype=torch.float16)
    for b in range(batch):
        g = _gen("cpu", stream_seed(seed, KIND_HIDDEN, 0, 0, 0, 1 + b))
        eps = torch.randn(tokens, hidden, generator=g, dtype=torch.float32)
        x = eps[0] / (1.0 - rho * rho) ** 0.5
        out[0, b] = x.to(torch.float16)
        for t in range(1, tokens):
            x = rho * x + eps[t]
            out[t, b] = x.to(torch.float16)
    return out


def layer_formats(shape: MoEShape) -> List[Tuple[int, int]]:
    """(bits, group) per layer.  Fixed-format configs repeat it; the mixed config draws,
    per layer, 2-bit group 16 or 3-bit group 64 from the seed (one draw per layer)."""
    if shape.bits:
        return [(shape.bits, shape.group)] * shape.layers
    g = _gen("cpu", stream_seed(shape.seed, KIND_FORMAT))
    draws = torch.randint(0, 2, (shape.layers,), generator=g)
    return [(2, 16) if int(d) == 0 else (3, 64) for d in draws]

"""CPU oracle for the MoE-offloading decode step.  TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 numpy written from the paper's description of the method
(arXiv 2312.17238).  It shares no code with the HIP path and must never be
imported by it; only tests, the smoke check and the bench's CPU-baseline leg
use it.

What follows the paper, and where:

* linear token-level gate, top-k selection of experts (Sec. 2.1; "both (2)
  active experts" of Mixtral, Sec. 4.1) -- `gate_logits`, `top_k`, `route`;
* group-wise low-bit weights with a scale and a zero point per group, the
  stored weight being (code - zero) * scale (Sec. 4.2) -- `dequantize`;
* an LRU cache of k experts per layer, the same k for every layer (Sec. 3.1,
  Sec. 3.3) -- `ExpertCacheSim`.  Sec. 3.1's sentence says the k "least"
  recently used experts are kept; that contradicts Sec. 3.3 ("replace the
  least recently used expert") and is read as a slip: the k most recently used
  stay, the least recently used one is evicted;
* speculative loading: the next layer's gate applied to the hidden state the
  current layer's gate saw, fetching the 1-2 most likely experts into
  temporary buffers that replace nothing until used (Sec. 3.2, Sec. 3.3) --
  `prefetch_scores`, `prefetch_guess`, `ExpertCacheSim.step`; its recall measured in
  isolation, 1, 2 and 10 layers ahead (Sec. 4.1) -- `speculative_recall`;
* "expert recall" = fraction of needed experts already on the device (Sec. 4.1)
  -- `CacheStats.recall`.

What the paper leaves open and the benchmark definition fixes: softmax over
all experts, then top-2, then renormalise the two weights to sum 1; ties go to
the lower expert index; SwiGLU experts w2(silu(w1 h) * (w3 h)) without biases;
matrices stored [out, in] with quantization groups along `in`; RMSNorm with
eps 1e-5 in front of the gate in the stacked configs; residual x + y.

Parity status: every function here is pinned by tests/test_oracle_*.py against
closed forms, brute force, library routines or invariants, except the absolute
tolerance on the FFN output, which only the benchmark definition fixes.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

HIT, PREFETCH_HIT, MISS = 0, 1, 2


# ----------------------------------------------------------------------------
# numerical definition
# ----------------------------------------------------------------------------

def rmsnorm(x_f16: np.ndarray, gamma_f16: np.ndarray, eps: float) -> np.ndarray:
    """h = fp16( x * (mean(x^2) + eps)^(-1/2) * gamma ), fp64 inside.  x: [..., H] fp16.

    eps is the fp32 value of the configuration promoted to fp64."""
    x = x_f16.astype(np.float64)
    g = gamma_f16.astype(np.float64)
    e = np.float64(np.float32(eps))
    ms = (x * x).sum(axis=-1, keepdims=True) / x.shape[-1]
    r = 1.0 / np.sqrt(ms + e)
    return (x * r * g).astype(np.float16)


def gate_logits(w_gate_f32: np.ndarray, h_f16: np.ndarray) -> np.ndarray:
    """z = W_g h in fp64 (Sec. 2.1: linear gating function).  W_g [E,H] fp32, h [H] fp16 -> [E]."""
    return w_gate_f32.astype(np.float64) @ h_f16.astype(np.float64)


def softmax(z: np.ndarray) -> np.ndarray:
    e = np.exp(z - z.max())
    return e / e.sum()


def top_k(z: Sequence[float], k: int) -> List[int]:
    """Indices of the k largest entries, largest first; equal values: lower index first.
    Asked for more than there are, it returns all of them in that order."""
    chosen: List[int] = []
    for _ in range(min(k, len(z))):
        best = -1
        for e in range(len(z)):
            if e in chosen:
                continue
            if best < 0 or z[e] > z[best]:
                best = e
        chosen.append(best)
    return chosen


def route(w_gate_f32: np.ndarray, h_f16: np.ndarray, k: int = 2) -> Tuple[List[int], np.ndarray, np.ndarray]:
    """(selected experts, their combine weights summing to 1, the logits) for one token."""
    z = gate_logits(w_gate_f32, h_f16)
    p = softmax(z)
    idx = top_k(z, k)
    w = p[idx] / p[idx].sum()
    return idx, w, z


def quantize_minmax(w_f32: np.ndarray, bits: int, group: int, zero_limit: Optional[float] = None):
    """Reference asymmetric min/max quantizer (fp32 arithmetic, fp16 scale and zero).

    Per group along the last axis: scale = fp16((max-min)/(2^bits-1)), 1 if that is 0;
    zero = fp16(-min/scale) (real valued); code = clip(rint(w/scale + zero), 0, 2^bits-1)
    with the rounded scale and zero.  Returns (codes u8 [out,in], scale f16 [out,in/g], zero f16).

    zero_limit (second level only): a group whose values are so close together, relative to their size,
    that |min/scale| would exceed it (and overflow fp16) is stored as a constant instead: scale = 1,
    zero = fp16(-min), all codes 0."""
    out_f, in_f = w_f32.shape
    qmax = np.float32((1 << bits) - 1)
    wg = w_f32.astype(np.float32).reshape(out_f, in_f // group, group)
    lo = wg.min(axis=2)
    hi = wg.max(axis=2)
    s16 = ((hi - lo) / qmax).astype(np.float16)
    s16[s16 == 0] = np.float16(1.0)
    if zero_limit is not None:
        s16[np.abs(lo / s16.astype(np.float32)) > np.float32(zero_limit)] = np.float16(1.0)
    sf = s16.astype(np.float32)
    z16 = (-lo / sf).astype(np.float16)
    zf = z16.astype(np.float32)
    q = np.clip(np.rint(wg / sf[:, :, None] + zf[:, :, None]), np.float32(0), qmax)
    return q.astype(np.uint8).reshape(out_f, in_f), s16, z16


def dequantize(codes_u8: np.ndarray, scale_f16: np.ndarray, zero_f16: np.ndarray, group: int) -> np.ndarray:
    """W^[r,c] = (q[r,c] - zero[r, c//g]) * scale[r, c//g] in fp64 (Sec. 4.2 format)."""
    s = np.repeat(scale_f16.astype(np.float64), group, axis=1)
    z = np.repeat(zero_f16.astype(np.float64), group, axis=1)
    return (codes_u8.astype(np.float64) - z) * s


META8_ZERO_LIMIT = 60000.0   # largest |zero| a run's fp16 pair may carry (fp16 overflows at 65520)


def quantize_meta8(scale_f16: np.ndarray, zero_f16: np.ndarray, scale_group: int):
    """Second level (Sec. 4.2, "scale group size"): per row, runs of `scale_group` consecutive groups (the
    whole row if it has fewer; a last run of a row may be shorter) quantize their fp16 scales, and separately
    their fp16 zeros, to 8 bits with the min/max rule of quantize_minmax.  Returns (scale codes u8, zero codes u8,
    meta f16 [out, runs, 4], groups per run) with meta[r, j] = (scale, zero) of the scale codes followed by
    (scale, zero) of the zero codes."""
    groups = scale_f16.shape[1]
    r = min(scale_group, groups)
    runs = -(-groups // r)

    def level2(v16):
        # a short last run is filled up with copies of its last value: its minimum and maximum stay what they are
        v = np.pad(v16.astype(np.float32), ((0, 0), (0, runs * r - groups)), mode="edge")
        q, s, z = quantize_minmax(v, 8, r, zero_limit=META8_ZERO_LIMIT)
        return q[:, :groups], s, z

    qs, ss, sz = level2(scale_f16)
    qz, zs, zz = level2(zero_f16)
    return qs, qz, np.stack([ss, sz, zs, zz], axis=2), r


def meta8_scale_zero(scale_u8: np.ndarray, zero_u8: np.ndarray, meta_f16: np.ndarray, run_len: int):
    """The per-group scale and zero a two-level matrix stands for, fp64:
    scale = (scale code - meta[..,1]) * meta[..,0], zero = (zero code - meta[..,3]) * meta[..,2],
    meta[:, j] belonging to groups j run_len .. j run_len + run_len - 1 of the row."""
    groups = scale_u8.shape[1]
    assert (meta_f16.shape[1] - 1) * run_len < groups <= meta_f16.shape[1] * run_len
    m = np.repeat(meta_f16.astype(np.float64), run_len, axis=1)[:, :groups]
    return (scale_u8.astype(np.float64) - m[:, :, 1]) * m[:, :, 0], (zero_u8.astype(np.float64) - m[:, :, 3]) * m[:, :, 2]


def dequantize_meta8(codes_u8: np.ndarray, scale_u8: np.ndarray, zero_u8: np.ndarray, meta_f16: np.ndarray,
                     run_len: int, group: int) -> np.ndarray:
    """W^[r,c] = (q[r,c] - zero[r, c//g]) * scale[r, c//g] with the two-level scale and zero, fp64."""
    s, z = meta8_scale_zero(scale_u8, zero_u8, meta_f16, run_len)
    return (codes_u8.astype(np.float64) - np.repeat(z, group, axis=1)) * np.repeat(s, group, axis=1)


def dequantize_any(matrix, group: int) -> np.ndarray:
    """(codes, scale f16, zero f16) or (codes, scale codes, zero codes, meta, groups per run)."""
    return dequantize(*matrix, group) if len(matrix) == 3 else dequantize_meta8(*matrix, group)


def silu(u: np.ndarray) -> np.ndarray:
    return u / (1.0 + np.exp(-u))


def expert_ffn(h_f16: np.ndarray, expert, group: int) -> np.ndarray:
    """y_e = W2^ ( silu(W1^ h) * (W3^ h) ), fp64.  expert = [(codes, scale, zero)] for w1, w3, w2
    (or the two-level form of dequantize_meta8)."""
    h = h_f16.astype(np.float64)
    w1 = dequantize_any(expert[0], group)
    w3 = dequantize_any(expert[1], group)
    w2 = dequantize_any(expert[2], group)
    a = silu(w1 @ h) * (w3 @ h)
    return w2 @ a


@dataclasses.dataclass
class BlockResult:
    h: np.ndarray          # fp16 [H] gate input
    idx: List[int]         # selected experts, best first
    w: np.ndarray          # fp64 [K] combine weights
    logits: np.ndarray     # fp64 [E]
    y: np.ndarray          # fp64 [H] block output before the residual add
    x_out: np.ndarray      # fp16 [H]


def moe_block(x_f16: np.ndarray, w_gate_f32: np.ndarray, experts, group: int, k: int = 2,
              gamma_f16: Optional[np.ndarray] = None, eps: float = 0.0,
              ffn=expert_ffn) -> BlockResult:
    """One token through one MoE block: (norm) -> gate -> top-k -> experts -> weighted sum -> residual.

    `experts[e]` = [(codes, scale, zero)] * 3.  `ffn` lets a caller substitute another
    implementation of the same expert definition (the C loop version for large shapes)."""
    h = rmsnorm(x_f16, gamma_f16, eps) if eps > 0.0 else x_f16
    idx, w, z = route(w_gate_f32, h, k)
    y = np.zeros(x_f16.shape[-1], dtype=np.float64)
    for j, e in enumerate(idx):
        y = y + w[j] * ffn(h, experts[e], group)
    x_out = (x_f16.astype(np.float64) + y).astype(np.float16)
    return BlockResult(h, idx, w, z, y, x_out)


# ----------------------------------------------------------------------------
# speculative prefetch predictor (Sec. 3.2)
# ----------------------------------------------------------------------------

def prefetch_scores(w_gate_next_f32: np.ndarray, h_f16: np.ndarray) -> np.ndarray:
    """Next layer's gate applied to the hidden states the current gate saw.
    h: [B,H] (or [H]); score_e = sum over the B tokens of softmax(W_g^{l+1} h_token)_e."""
    hb = np.atleast_2d(h_f16)
    s = np.zeros(w_gate_next_f32.shape[0], dtype=np.float64)
    for t in range(hb.shape[0]):
        s = s + softmax(gate_logits(w_gate_next_f32, hb[t]))
    return s


def prefetch_guess(scores: np.ndarray, m: int) -> List[int]:
    """The m most likely next-layer experts, most likely first, ties to the lower index."""
    return top_k(list(scores), m)


def speculative_recall(routing, h_f16: np.ndarray, gates: Sequence[np.ndarray], ahead: int, m: int) -> Tuple[int, int]:
    """Speculative loading in isolation (Sec. 4.1, Fig. 2 right): for every token t and layer l, guess the experts
    of layer l+ahead by applying THAT layer's gate to the hidden state layer l's gate saw, keep the m most likely,
    and count how many of the experts layer l+ahead really selected were among them.

    routing[t][l]: experts selected for token t at layer l; h_f16[t][l]: [H] gate input of layer l; gates[l]: [E,H].
    Returns (guessed and needed, needed); the recall is their ratio, 1.0 when every active expert was guessed.
    ahead = 0 guesses a layer from its own gate input, which finds min(m, K) of its K experts by construction."""
    got = need = 0
    for t in range(len(routing)):
        for l in range(len(gates) - ahead):
            guess = prefetch_guess(prefetch_scores(gates[l + ahead], h_f16[t][l]), m)
            actual = routing[t][l + ahead]
            got += len(set(guess) & set(actual))
            need += len(actual)
    return got, need


# ----------------------------------------------------------------------------
# discrete simulation of the expert cache and the staging buffers (Sec. 3.1, 3.3)
# ----------------------------------------------------------------------------

@dataclasses.dataclass
class CacheStats:
    needed: int = 0
    hits: int = 0
    prefetch_hits: int = 0
    misses: int = 0
    evictions: int = 0
    spec_issued: int = 0
    spec_wasted: int = 0
    steps: int = 0

    @property
    def recall(self) -> float:
        """Sec. 4.1: fraction of needed experts that were already on the device."""
        return (self.hits + self.prefetch_hits) / self.needed if self.needed else 0.0


@dataclasses.dataclass
class Access:
    expert: int
    status: int
    slot: int
    victim: int  # evicted expert id, -1 if the slot was empty


class ExpertCacheSim:
    """L layers, k slots each, b staging buffers shared by all layers.

    Each slot holds an expert id (or -1) and a recency stamp from one global
    clock.  `staged[l]` is the set of speculatively loaded experts waiting for
    layer l; they live outside the cache, touch no stamp and evict nothing
    until layer l actually uses them (Sec. 3.3).
    """

    def __init__(self, layers: int, n_experts: int, k: int, b: int = 4, warm: bool = False):
        self.L, self.E, self.k, self.b = layers, n_experts, k, b
        self.slot_expert = [[-1] * k for _ in range(layers)]
        self.slot_stamp = [[0] * k for _ in range(layers)]
        self.staged: List[List[int]] = [[] for _ in range(layers)]
        self.clock = 0
        self.stats = [CacheStats() for _ in range(layers)]
        if warm:
            for l in range(layers):
                for s in range(min(k, n_experts)):
                    self.clock += 1
                    self.slot_expert[l][s] = s
                    self.slot_stamp[l][s] = self.clock

    def staged_total(self) -> int:
        return sum(len(p) for p in self.staged)

    def contents(self, l: int) -> List[int]:
        return sorted(e for e in self.slot_expert[l] if e >= 0)

    def step(self, l: int, selected: Sequence[Sequence[int]],
             guess: Optional[Sequence[int]] = None) -> Tuple[List[Access], List[Tuple[int, bool]]]:
        """One decode step of layer l.

        selected: per token, its top-k experts.  guess: ordered speculative guess
        for layer l+1 (None or empty: no prefetch).  Returns the accesses in the
        order they touch the cache, and [(guessed expert, copy issued?)].
        """
        st = self.stats[l]
        st.steps += 1
        needed = sorted({int(e) for tok in selected for e in tok})
        resident = [e for e in needed if e in self.slot_expert[l]]
        absent = [e for e in needed if e not in self.slot_expert[l]]
        trace: List[Access] = []
        for e in resident:
            s = self.slot_expert[l].index(e)
            self.clock += 1
            self.slot_stamp[l][s] = self.clock
            st.hits += 1
            trace.append(Access(e, HIT, s, -1))
        for e in absent:
            status = PREFETCH_HIT if e in self.staged[l] else MISS
            if -1 in self.slot_expert[l]:
                s = self.slot_expert[l].index(-1)
                victim = -1
            else:
                s = min(range(self.k), key=lambda i: self.slot_stamp[l][i])
                victim = self.slot_expert[l][s]
                st.evictions += 1
            self.slot_expert[l][s] = e
            self.clock += 1
            self.slot_stamp[l][s] = self.clock
            if status == PREFETCH_HIT:
                st.prefetch_hits += 1
            else:
                st.misses += 1
            trace.append(Access(e, status, s, victim))
        st.needed += len(needed)
        st.spec_wasted += len([e for e in self.staged[l] if e not in needed])
        self.staged[l] = []
        decisions: List[Tuple[int, bool]] = []
        if guess and l + 1 < self.L:
            for e in guess:
                e = int(e)
                issue = (e not in self.slot_expert[l + 1] and e not in self.staged[l + 1]
                         and self.staged_total() < self.b)
                if issue:
                    self.staged[l + 1].append(e)
                    self.stats[l + 1].spec_issued += 1
                decisions.append((e, issue))
        return trace, decisions


class SwapPlacement:
    """Where every expert of one layer lives when host memory cannot hold them all (Sec. 3.3).

    An expert is in exactly one buffer: on the device (one of the k cache slots) or in one of the
    host buffers.  Loading an expert onto the device sends the evicted one back to the host, so the
    counts on both sides never change.  Reading of what the paper leaves open: there are
    E - k + 1 host buffers, one of them empty ("spare"); the evicted expert is written into the
    spare, and the buffer the loaded expert came from becomes the spare -- so the write never has to
    wait for the load to finish reading.  Experts 0..k-1 start on the device, expert e >= k starts in
    host buffer e - k, the spare is buffer E - k.
    """

    def __init__(self, n_experts: int, k: int):
        self.E, self.k = n_experts, k
        self.host_buf_of = [-1 if e < k else e - k for e in range(n_experts)]
        self.spare = n_experts - k
        self.writebacks = 0

    def apply(self, accesses: Sequence[Access]) -> None:
        """Follow the accesses of one step (as ExpertCacheSim.step returns them, warm-started)."""
        for a in accesses:
            if a.status == HIT:
                continue
            if a.victim < 0:
                raise ValueError("swap placement needs a full cache: every load evicts")
            came_from = self.host_buf_of[a.expert]
            if came_from < 0 or self.host_buf_of[a.victim] >= 0:
                raise ValueError("placement and cache trace disagree")
            self.host_buf_of[a.victim] = self.spare
            self.spare = came_from
            self.host_buf_of[a.expert] = -1
            self.writebacks += 1

    def on_device(self) -> List[int]:
        return sorted(e for e in range(self.E) if self.host_buf_of[e] < 0)

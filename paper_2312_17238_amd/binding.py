"""ctypes binding of libmoe_offload.so: argument marshalling only.

Function names and arguments mirror include/moe_offload.h one to one.  Every step of the
decode path runs inside the library; PyTorch appears here only as the owner of device
memory, pinned host memory and streams (`Engine` below).
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmoe_offload.so")

MOE_MAX_EXPERTS, MOE_MAX_TOPK, MOE_MAX_BATCH, MOE_MAX_GUESS = 16, 4, 1024, 4
MOE_OK, MOE_EINVAL, MOE_ESTATE, MOE_ENOMEM, MOE_EHIP = 0, -1, -2, -3, -4
MOE_HIT, MOE_PREFETCH_HIT, MOE_MISS = 0, 1, 2
MOE_CTX_HOST_ONLY = 1
MOE_LAYER_NO_CACHE = 1
MOE_LAYER_SWAP = 2

EXPORTS = [
    "moe_expert_blob_bytes", "moe_expert_blob_bytes_2level", "moe_ctx_dev_bytes", "moe_layer_dev_bytes", "moe_layer_host_bytes",
    "moe_ctx_create", "moe_ctx_destroy", "moe_layer_create", "moe_layer_destroy",
    "moe_layer_load_expert", "moe_layer_load_expert_2level", "moe_layer_peek_weight", "moe_layer_peek_run_meta", "moe_layer_step", "moe_layer_step_noalloc", "moe_layer_prefetch",
    "moe_stack_step", "moe_layer_resolve", "moe_layer_stats", "moe_layer_cache_state", "moe_layer_placement",
    "moe_layer_reset", "moe_ctx_read_y", "moe_ctx_profile_enable", "moe_ctx_profile_read", "moe_ctx_profile_timeline", "moe_ctx_set_option", "moe_probe_bandwidth", "moe_layer_set_prefetch", "moe_layer_set_flags", "moe_last_error", "moe_last_hip_error",
]


class CtxConfig(C.Structure):
    _fields_ = [("n_staging", C.c_int32), ("max_batch", C.c_int32), ("max_hidden", C.c_int32),
                ("max_ffn", C.c_int32), ("max_top_k", C.c_int32), ("flags", C.c_int32),
                ("max_expert_bytes", C.c_uint64)]


class LayerConfig(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("ffn", C.c_int32), ("n_experts", C.c_int32), ("top_k", C.c_int32),
                ("bits", C.c_int32), ("group", C.c_int32), ("cache_slots", C.c_int32), ("prefetch_m", C.c_int32),
                ("rms_eps", C.c_float), ("init_policy", C.c_int32), ("flags", C.c_int32), ("scale_group", C.c_int32)]


class Access(C.Structure):
    _fields_ = [("expert", C.c_int32), ("status", C.c_int32), ("slot", C.c_int32), ("victim", C.c_int32)]


class StepTrace(C.Structure):
    _fields_ = [("batch", C.c_int32), ("top_k", C.c_int32), ("n_experts", C.c_int32),
                ("expert_idx", C.c_int32 * (MOE_MAX_BATCH * MOE_MAX_TOPK)),
                ("expert_w", C.c_float * (MOE_MAX_BATCH * MOE_MAX_TOPK)),
                ("logits", C.c_double * (MOE_MAX_BATCH * MOE_MAX_EXPERTS)),
                ("n_access", C.c_int32),
                ("access", Access * MOE_MAX_EXPERTS),
                ("n_guess", C.c_int32),
                ("guess_expert", C.c_int32 * MOE_MAX_GUESS),
                ("guess_issued", C.c_int32 * MOE_MAX_GUESS),
                ("guess_score", C.c_double * MOE_MAX_EXPERTS)]

    def routing(self) -> List[List[int]]:
        k = self.top_k
        return [[self.expert_idx[b * k + j] for j in range(k)] for b in range(self.batch)]

    def weights(self) -> List[List[float]]:
        k = self.top_k
        return [[self.expert_w[b * k + j] for j in range(k)] for b in range(self.batch)]

    def accesses(self):
        return [(a.expert, a.status, a.slot, a.victim) for a in self.access[: self.n_access]]

    def guesses(self):
        return [(self.guess_expert[i], bool(self.guess_issued[i])) for i in range(self.n_guess)]


class Stats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("steps", "needed", "hits", "prefetch_hits", "misses", "evictions",
                                          "spec_issued", "spec_wasted", "bytes_h2d_demand", "bytes_h2d_spec",
                                          "bytes_d2h_writeback", "steps_device_routed")]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class ProfileEntry(C.Structure):
    _fields_ = [("launches", C.c_uint64), ("bytes", C.c_uint64), ("total_ms", C.c_double)]


class Profile(C.Structure):
    _fields_ = [("gate", ProfileEntry), ("w13", ProfileEntry), ("w2", ProfileEntry), ("copy", ProfileEntry),
                ("ffn", ProfileEntry), ("writeback", ProfileEntry)]

    def as_dict(self):
        return {k: {"launches": int(getattr(self, k).launches), "bytes": int(getattr(self, k).bytes),
                    "total_ms": float(getattr(self, k).total_ms)} for k, _ in self._fields_}


class MoeError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"moe_offload error {code}: {msg}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """Load the built library.  There is no fallback: without it the package cannot compute."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2312_17238_amd.build` "
                          "(or __graft_entry__.build()); there is no CPU fallback")
    L = C.CDLL(LIB_PATH)
    vp, i32, u64 = C.c_void_p, C.c_int32, C.c_uint64
    L.moe_expert_blob_bytes.restype = u64
    L.moe_expert_blob_bytes.argtypes = [i32, i32, i32, i32]
    L.moe_expert_blob_bytes_2level.restype = u64
    L.moe_expert_blob_bytes_2level.argtypes = [i32, i32, i32, i32, i32]
    L.moe_layer_load_expert_2level.argtypes = [vp, i32, i32, vp, vp, vp, vp]
    L.moe_layer_peek_run_meta.argtypes = [vp, i32, i32, i32, i32, C.POINTER(C.c_uint16)]
    L.moe_ctx_dev_bytes.restype = u64
    L.moe_ctx_dev_bytes.argtypes = [C.POINTER(CtxConfig)]
    L.moe_layer_dev_bytes.restype = u64
    L.moe_layer_dev_bytes.argtypes = [vp, C.POINTER(LayerConfig)]
    L.moe_layer_host_bytes.restype = u64
    L.moe_layer_host_bytes.argtypes = [C.POINTER(LayerConfig)]
    L.moe_ctx_create.argtypes = [C.POINTER(CtxConfig), vp, u64, vp, vp, C.POINTER(vp)]
    L.moe_ctx_destroy.argtypes = [vp]
    L.moe_layer_create.argtypes = [vp, C.POINTER(LayerConfig), vp, vp, vp, vp, C.POINTER(vp)]
    L.moe_layer_destroy.argtypes = [vp]
    L.moe_layer_load_expert.argtypes = [vp, i32, i32, vp, vp, vp]
    L.moe_layer_peek_weight.argtypes = [vp, i32, i32, i32, i32, C.POINTER(C.c_uint8), C.POINTER(C.c_uint16),
                                        C.POINTER(C.c_uint16)]
    L.moe_layer_step.argtypes = [vp, vp, vp, i32, vp, vp, C.POINTER(StepTrace)]
    L.moe_layer_step_noalloc.argtypes = [vp, vp, vp, i32, vp, vp, C.POINTER(StepTrace)]
    L.moe_layer_prefetch.argtypes = [vp, vp, i32, C.POINTER(StepTrace)]
    L.moe_stack_step.argtypes = [C.POINTER(vp), i32, vp, i32, vp, C.POINTER(StepTrace)]
    L.moe_layer_resolve.argtypes = [vp, vp, C.POINTER(i32), i32, C.POINTER(C.c_double), C.POINTER(StepTrace)]
    L.moe_layer_stats.argtypes = [vp, C.POINTER(Stats)]
    L.moe_layer_cache_state.argtypes = [vp, C.POINTER(i32), C.POINTER(u64), C.POINTER(i32), C.POINTER(i32)]
    L.moe_layer_placement.argtypes = [vp, C.POINTER(i32), C.POINTER(i32)]
    L.moe_layer_reset.argtypes = [vp]
    L.moe_ctx_read_y.argtypes = [vp, i32, i32, vp]
    L.moe_ctx_profile_enable.argtypes = [vp, i32]
    L.moe_ctx_profile_read.argtypes = [vp, C.POINTER(Profile)]
    L.moe_ctx_profile_timeline.argtypes = [vp, i32, C.POINTER(C.c_double), C.POINTER(C.c_double), i32, C.POINTER(i32)]
    L.moe_ctx_set_option.argtypes = [vp, C.c_char_p, i32]
    L.moe_probe_bandwidth.argtypes = [vp, vp, u64, i32, i32, vp, C.POINTER(C.c_double)]
    L.moe_layer_set_prefetch.argtypes = [vp, i32]
    L.moe_layer_set_flags.argtypes = [vp, i32]
    L.moe_last_error.restype = C.c_char_p
    L.moe_last_hip_error.restype = i32
    for name in EXPORTS:
        fn = getattr(L, name)
        if fn.restype is C.c_int:
            fn.restype = i32
    _lib = L
    return L


def check(rc: int) -> None:
    if rc != MOE_OK:
        raise MoeError(rc, lib().moe_last_error().decode(errors="replace"))


# --------------------------------------------------------------------------------------------
# thin wrappers, same names as the C entry points
# --------------------------------------------------------------------------------------------

def moe_expert_blob_bytes(hidden: int, ffn: int, bits: int, group: int, scale_group: int = 0) -> int:
    if scale_group:
        return int(lib().moe_expert_blob_bytes_2level(hidden, ffn, bits, group, scale_group))
    return int(lib().moe_expert_blob_bytes(hidden, ffn, bits, group))


def moe_ctx_dev_bytes(cfg: CtxConfig) -> int:
    return int(lib().moe_ctx_dev_bytes(C.byref(cfg)))


def moe_layer_dev_bytes(ctx, cfg: LayerConfig) -> int:
    return int(lib().moe_layer_dev_bytes(ctx, C.byref(cfg)))


def moe_layer_host_bytes(cfg: LayerConfig) -> int:
    return int(lib().moe_layer_host_bytes(C.byref(cfg)))


def moe_ctx_create(cfg: CtxConfig, dev_arena: int, dev_arena_bytes: int, compute_stream: int, copy_stream: int):
    out = C.c_void_p()
    check(lib().moe_ctx_create(C.byref(cfg), dev_arena, dev_arena_bytes, compute_stream, copy_stream, C.byref(out)))
    return out


def moe_ctx_destroy(ctx) -> None:
    check(lib().moe_ctx_destroy(ctx))


def moe_layer_create(ctx, cfg: LayerConfig, gate_w_host: int, rms_gamma_host: Optional[int], dev_mem: int,
                     pinned_host_mem: int):
    out = C.c_void_p()
    check(lib().moe_layer_create(ctx, C.byref(cfg), gate_w_host, rms_gamma_host, dev_mem, pinned_host_mem, C.byref(out)))
    return out


def moe_layer_destroy(layer) -> None:
    check(lib().moe_layer_destroy(layer))


def moe_layer_load_expert(layer, expert: int, matrix: int, codes: int, scale: int, zero: int) -> None:
    check(lib().moe_layer_load_expert(layer, expert, matrix, codes, scale, zero))


def moe_layer_load_expert_2level(layer, expert: int, matrix: int, codes: int, scale_code: int, zero_code: int,
                                 run_meta: int) -> None:
    check(lib().moe_layer_load_expert_2level(layer, expert, matrix, codes, scale_code, zero_code, run_meta))


def moe_layer_peek_run_meta(layer, expert: int, matrix: int, row: int, col: int):
    m = (C.c_uint16 * 4)()
    check(lib().moe_layer_peek_run_meta(layer, expert, matrix, row, col, m))
    return tuple(m)


def moe_layer_peek_weight(layer, expert: int, matrix: int, row: int, col: int):
    c, s, z = C.c_uint8(), C.c_uint16(), C.c_uint16()
    check(lib().moe_layer_peek_weight(layer, expert, matrix, row, col, C.byref(c), C.byref(s), C.byref(z)))
    return c.value, s.value, z.value


def moe_layer_step(layer, next_layer, x_in_dev: int, batch: int, x_out_dev: int, h_out_dev: Optional[int] = None,
                   trace: Optional[StepTrace] = None) -> None:
    check(lib().moe_layer_step(layer, next_layer, x_in_dev, batch, x_out_dev, h_out_dev,
                               C.byref(trace) if trace is not None else None))


def moe_layer_step_noalloc(layer, next_layer, x_in_dev: int, batch: int, x_out_dev: int, h_out_dev: Optional[int] = None,
                           trace: Optional[StepTrace] = None) -> None:
    check(lib().moe_layer_step_noalloc(layer, next_layer, x_in_dev, batch, x_out_dev, h_out_dev,
                                       C.byref(trace) if trace is not None else None))


def moe_layer_prefetch(layer, h_dev: int, batch: int, trace: Optional[StepTrace] = None) -> None:
    check(lib().moe_layer_prefetch(layer, h_dev, batch, C.byref(trace) if trace is not None else None))


def moe_stack_step(layers: Sequence, x_in_dev: int, batch: int, x_out_dev: int, traces=None) -> None:
    arr = (C.c_void_p * len(layers))(*[l.value if isinstance(l, C.c_void_p) else l for l in layers])
    check(lib().moe_stack_step(arr, len(layers), x_in_dev, batch, x_out_dev, traces))


def moe_layer_resolve(layer, next_layer, expert_idx: Sequence[int], batch: int, guess_score=None,
                      trace: Optional[StepTrace] = None) -> None:
    idx = (C.c_int32 * len(expert_idx))(*expert_idx)
    gs = (C.c_double * len(guess_score))(*guess_score) if guess_score is not None else None
    check(lib().moe_layer_resolve(layer, next_layer, idx, batch, gs, C.byref(trace) if trace is not None else None))


def moe_layer_stats(layer) -> Stats:
    s = Stats()
    check(lib().moe_layer_stats(layer, C.byref(s)))
    return s


def moe_layer_cache_state(layer, k: int):
    se, ss = (C.c_int32 * k)(), (C.c_uint64 * k)()
    st, n = (C.c_int32 * MOE_MAX_EXPERTS)(), C.c_int32()
    check(lib().moe_layer_cache_state(layer, se, ss, st, C.byref(n)))
    return list(se), list(ss), list(st)[: n.value]


def moe_layer_placement(layer, n_experts: int):
    """(host buffer of each expert or -1 while it is on the device, spare host buffer)."""
    hb, sp = (C.c_int32 * n_experts)(), C.c_int32()
    check(lib().moe_layer_placement(layer, hb, C.byref(sp)))
    return list(hb), sp.value


def moe_layer_reset(layer) -> None:
    check(lib().moe_layer_reset(layer))


def moe_ctx_read_y(ctx, batch: int, hidden: int, y_host: int) -> None:
    check(lib().moe_ctx_read_y(ctx, batch, hidden, y_host))


def moe_ctx_profile_enable(ctx, on: bool) -> None:
    check(lib().moe_ctx_profile_enable(ctx, 1 if on else 0))


def moe_ctx_profile_timeline(ctx, kind: int, cap: int = 1 << 16):
    """[(start ms, stop ms)] of the launches of one kind recorded since profiling was switched on."""
    a, b, n = (C.c_double * cap)(), (C.c_double * cap)(), C.c_int32()
    check(lib().moe_ctx_profile_timeline(ctx, kind, a, b, cap, C.byref(n)))
    return [(a[i], b[i]) for i in range(min(cap, n.value))]


def moe_ctx_profile_read(ctx) -> Profile:
    p = Profile()
    check(lib().moe_ctx_profile_read(ctx, C.byref(p)))
    return p


def moe_ctx_set_option(ctx, name: str, value: int) -> None:
    check(lib().moe_ctx_set_option(ctx, name.encode(), value))


def moe_probe_bandwidth(src_dev: int, dst_dev: Optional[int], nbytes: int, blocks: int, iters: int, stream: int) -> float:
    """Average milliseconds per launch of the plain read (dst_dev None) or copy probe kernel."""
    ms = C.c_double()
    check(lib().moe_probe_bandwidth(src_dev, dst_dev, nbytes, blocks, iters, stream, C.byref(ms)))
    return ms.value


def moe_layer_set_prefetch(layer, m: int) -> None:
    check(lib().moe_layer_set_prefetch(layer, m))


def moe_layer_set_flags(layer, flags: int) -> None:
    check(lib().moe_layer_set_flags(layer, flags))

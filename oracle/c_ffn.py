"""ctypes wrapper over the C oracle's expert FFN (test infrastructure only)."""
from __future__ import annotations

import ctypes

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(_build.build())
        _lib.moe_oracle_expert_ffn.restype = ctypes.c_int
        _lib.moe_oracle_expert_ffn.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p] * 11
        _lib.moe_oracle_expert_ffn_f64meta.restype = ctypes.c_int
        _lib.moe_oracle_expert_ffn_f64meta.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p] * 11
        _lib.moe_oracle_threads.restype = ctypes.c_int
    return _lib


def threads() -> int:
    return int(_load().moe_oracle_threads())


def _p(a: np.ndarray, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == dtype, (a.dtype, dtype)
    return a


def expert_ffn(h_f16: np.ndarray, expert, group: int) -> np.ndarray:
    """Same contract as moe_oracle.expert_ffn, computed by the plain C loops."""
    lib = _load()
    if len(expert[0]) == 5:
        return _expert_ffn_meta8(lib, h_f16, expert, group)
    (q1, s1, z1), (q3, s3, z3), (q2, s2, z2) = expert
    F, H = q1.shape
    assert q3.shape == (F, H) and q2.shape == (H, F)
    keep = [_p(h_f16, np.float16)]
    for q, s, z in ((q1, s1, z1), (q3, s3, z3), (q2, s2, z2)):
        keep += [_p(q, np.uint8), _p(s, np.float16), _p(z, np.float16)]
    y = np.empty(H, dtype=np.float64)
    rc = lib.moe_oracle_expert_ffn(H, F, group, *[a.ctypes.data for a in keep], y.ctypes.data)
    if rc != 0:
        raise ValueError("moe_oracle_expert_ffn rejected its arguments")
    return y


def _expert_ffn_meta8(lib, h_f16: np.ndarray, expert, group: int) -> np.ndarray:
    """Two-level experts [(codes, scale codes, zero codes, meta, groups per run)]: the second level is evaluated by the numpy
    oracle's definition (a few numbers per row), the loops over the weights run in C."""
    from . import moe_oracle as O
    F, H = expert[0][0].shape
    keep = [_p(h_f16, np.float16)]
    for q, qs, qz, meta, run_len in expert:
        s, z = O.meta8_scale_zero(qs, qz, meta, run_len)
        keep += [_p(q, np.uint8), _p(s, np.float64), _p(z, np.float64)]
    y = np.empty(H, dtype=np.float64)
    rc = lib.moe_oracle_expert_ffn_f64meta(H, F, group, *[a.ctypes.data for a in keep], y.ctypes.data)
    if rc != 0:
        raise ValueError("moe_oracle_expert_ffn_f64meta rejected its arguments")
    return y

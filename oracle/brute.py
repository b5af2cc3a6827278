"""ctypes loader for the brute-force C twin (test infrastructure; see skv_oracle_brute.c)."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "skv_oracle_brute.c")
_LIB = os.path.join(_HERE, "libskv_oracle_brute.so")


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.skvo_slot_map.restype = ctypes.c_int
        _lib.skvo_attention.restype = ctypes.c_int
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def slot_map(route):
    route = np.ascontiguousarray(route, dtype=np.int32)
    slot = np.zeros(len(route), dtype=np.int32)
    n = ctypes.c_int(0)
    rc = _load().skvo_slot_map(_p(route, ctypes.c_int), len(route), _p(slot, ctypes.c_int), ctypes.byref(n))
    if rc:
        raise ValueError("invalid route")
    return slot.tolist(), n.value


def attention(kc, vc, slot, q, q_lens, kv_lens, scale):
    """kc, vc: [slots][B][ctx][Hkv][D] float64; q: [B][S][Hq][D] float64 -> out like q."""
    kc = np.ascontiguousarray(kc, dtype=np.float64)
    vc = np.ascontiguousarray(vc, dtype=np.float64)
    q = np.ascontiguousarray(q, dtype=np.float64)
    q_lens = np.ascontiguousarray(q_lens, dtype=np.int32)
    kv_lens = np.ascontiguousarray(kv_lens, dtype=np.int32)
    _, B, ctx, hkv, d = kc.shape
    _, S, hq, _ = q.shape
    out = np.zeros_like(q)
    dp = ctypes.c_double
    rc = _load().skvo_attention(_p(kc, dp), _p(vc, dp), B, ctx, hkv, d, int(slot), _p(q, dp), S, hq,
                                _p(q_lens, ctypes.c_int), _p(kv_lens, ctypes.c_int),
                                ctypes.c_double(scale), _p(out, dp))
    if rc:
        raise ValueError(f"skvo_attention failed with {rc}")
    return out

"""ctypes front end of the C oracle (TEST INFRASTRUCTURE ONLY).

`attn(q, k, v, causal, scale, algo, rows)` evaluates attention in fp64 on the
CPU for torch CPU tensors of any of the three storage dtypes; the values are
widened exactly to float and then to double inside the C code.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

from . import build as _build

ALGO = {"definition": 0, "alg1": 1, "alg2": 2, "alg3": 3}

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.LIB if os.path.exists(_build.LIB) else _build.build()
        lib = ctypes.CDLL(path)
        lib.oracle_attn.restype = ctypes.c_int
        lib.oracle_attn.argtypes = [
            ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int, ctypes.c_float, ctypes.c_void_p, ctypes.c_long]
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_attn_state.restype = ctypes.c_int
        lib.oracle_attn_state.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int, ctypes.c_int, ctypes.c_float]
        lib.oracle_skip_stats.restype = ctypes.c_int
        lib.oracle_skip_stats.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_float,
            ctypes.c_float, ctypes.c_float, ctypes.c_void_p]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _as_f32(x: torch.Tensor) -> np.ndarray:
    if x.device.type != "cpu":
        raise ValueError("the oracle takes CPU tensors")
    return np.ascontiguousarray(x.detach().to(torch.float32).numpy())


def attn(q, k, v, causal: bool, scale: float, algo: str = "definition", rows=None) -> np.ndarray:
    """fp64 attention.  q: [B,Hq,Lq,d], k/v: [B,Hkv,Lk,d].

    rows=None -> array [B,Hq,Lq,d]; rows = int array [n,3] of (b,h,i) ->
    array [n,d] holding only those query rows.
    """
    lib = _load()
    qf, kf, vf = _as_f32(q), _as_f32(k), _as_f32(v)
    B, Hq, Lq, d = qf.shape
    Bk, Hkv, Lk, dk = kf.shape
    if vf.shape != kf.shape or Bk != B or dk != d:
        raise ValueError("shape mismatch")
    if rows is None:
        out = np.empty((B, Hq, Lq, d), dtype=np.float64)
        rows_p, n = None, 0
    else:
        rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int32).reshape(-1, 3))
        out = np.empty((rows.shape[0], d), dtype=np.float64)
        rows_p, n = rows.ctypes.data, rows.shape[0]
    rc = lib.oracle_attn(ALGO[algo], qf.ctypes.data, kf.ctypes.data, vf.ctypes.data,
                         out.ctypes.data, B, Hq, Hkv, Lq, Lk, d, int(bool(causal)),
                         float(np.float32(scale)), rows_p, n)
    if rc != 0:
        raise ValueError("oracle_attn rejected its arguments")
    return out


def skip_stats(q, k, causal: bool, scale: float, lo: float = -6.0, hi: float = 11.0):
    """(steps, low, high) of the static skip rule of Sec. III-C over all query rows: steps
    i >= 2 of each row's visible keys, those with s_i - s_{i-1} <= lo, those with >= hi.
    Scores in the fixed fp32 arithmetic that skip_oracle.c documents."""
    lib = _load()
    qf, kf = _as_f32(q), _as_f32(k)
    B, Hq, Lq, d = qf.shape
    Bk, Hkv, Lk, dk = kf.shape
    if Bk != B or dk != d:
        raise ValueError("shape mismatch")
    counts = np.zeros(3, dtype=np.uint64)
    rc = lib.oracle_skip_stats(qf.ctypes.data, kf.ctypes.data, B, Hq, Hkv, Lq, Lk, d,
                               int(bool(causal)), float(np.float32(scale)),
                               float(np.float32(lo)), float(np.float32(hi)), counts.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_skip_stats rejected its arguments")
    return int(counts[0]), int(counts[1]), int(counts[2])


def attn_state(q, k, v, causal: bool, scale: float, state_in=None, shift=None) -> np.ndarray:
    """Alg. 3 over this call's keys, continuing from `state_in` (fp64 array [B,Hq,Lq,d+2] of
    (o, s_last, ln w_last) per row, or None).  Returns the literal state in the same layout.
    causal: key j visible to query i iff j <= i + shift (default Lk - Lq)."""
    lib = _load()
    qf, kf, vf = _as_f32(q), _as_f32(k), _as_f32(v)
    B, Hq, Lq, d = qf.shape
    Bk, Hkv, Lk, dk = kf.shape
    if vf.shape != kf.shape or Bk != B or dk != d:
        raise ValueError("shape mismatch")
    out = np.empty((B, Hq, Lq, d + 2), dtype=np.float64)
    sin_p = None
    if state_in is not None:
        state_in = np.ascontiguousarray(state_in, dtype=np.float64)
        if state_in.shape != out.shape:
            raise ValueError("state_in must be [B,Hq,Lq,d+2]")
        sin_p = state_in.ctypes.data
    sh = Lk - Lq if shift is None else int(shift)
    rc = lib.oracle_attn_state(qf.ctypes.data, kf.ctypes.data, vf.ctypes.data, sin_p,
                               out.ctypes.data, B, Hq, Hkv, Lq, Lk, d, int(bool(causal)), sh,
                               float(np.float32(scale)))
    if rc != 0:
        raise ValueError("oracle_attn_state rejected its arguments")
    return out

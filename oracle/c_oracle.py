"""ctypes front-end for the plain-C oracle (oracle/snapkv_oracle.c).  Test infrastructure only."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "snapkv_oracle.c")
LIB = os.path.join(_HERE, "libsnapkv_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over KV heads; no fast-math)."""
    # Compiles only when asked to or when no library is there: a benchmark or test process must
    # not start a compiler on its own (file times do not survive every way of copying a tree).
    if force or not os.path.exists(LIB):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", LIB, SRC, "-lm"])
    return LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(LIB)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        L.snapkv_oracle_threads.restype = i32
        L.snapkv_oracle_pooled_scores.restype = i32
        L.snapkv_oracle_pooled_scores.argtypes = [vp, vp, i32, i64, i32, i32, i32, i32, i32, i32, vp]
        L.snapkv_oracle_compress.restype = i64
        L.snapkv_oracle_compress.argtypes = [vp, vp, vp, i32, i64, i32, i32, i32, i32, i32, i32,
                                             i64, vp, vp, vp, vp]
        _lib = L
    return _lib


def threads() -> int:
    return int(lib().snapkv_oracle_threads())


def _storage(a: np.ndarray):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return a, 1
    if a.dtype == np.float32:
        return a, 0
    raise TypeError("storage must be float32 or uint16 (bf16 bits)")


def pooled_scores(q_win, k, W, pool_kind, p) -> np.ndarray:
    q_win, b1 = _storage(q_win)
    k, b2 = _storage(k)
    assert b1 == b2
    Hq, Wq, D = q_win.shape
    Hkv, L, _ = k.shape
    assert Wq == W
    out = np.empty((Hkv, L - W), dtype=np.float64)
    rc = lib().snapkv_oracle_pooled_scores(q_win.ctypes.data, k.ctypes.data, b1, L, Hq, Hkv, D, W,
                                           pool_kind, p, out.ctypes.data)
    if rc:
        raise ValueError(f"snapkv_oracle_pooled_scores failed: {rc}")
    return out


def compress(q_win, k, v, W, pool_kind, p, C):
    q_win, b1 = _storage(q_win)
    k, b2 = _storage(k)
    v, b3 = _storage(v)
    assert b1 == b2 == b3
    Hq, Wq, D = q_win.shape
    Hkv, L, _ = k.shape
    assert Wq == W
    out_k = np.zeros((Hkv, C, D), dtype=k.dtype)
    out_v = np.zeros((Hkv, C, D), dtype=v.dtype)
    out_idx = np.zeros((Hkv, C), dtype=np.int64)
    score = np.zeros((Hkv, max(L - W, 0)), dtype=np.float64) if L > C else None
    kept = lib().snapkv_oracle_compress(q_win.ctypes.data, k.ctypes.data, v.ctypes.data, b1, L, Hq,
                                        Hkv, D, W, pool_kind, p, C, out_k.ctypes.data,
                                        out_v.ctypes.data, out_idx.ctypes.data,
                                        score.ctypes.data if score is not None else None)
    if kept < 0:
        raise ValueError(f"snapkv_oracle_compress failed: {kept}")
    return out_k[:, :kept], out_v[:, :kept], out_idx[:, :kept], int(kept), score

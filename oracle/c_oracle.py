"""ctypes wrapper around the plain-C oracle (oracle/topk_attn_oracle.c).

TEST INFRASTRUCTURE: used by tests, the smoke check and the benchmark's
cpu_baseline leg only.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "topk_attn_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

F32, F16, BF16 = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (host code only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        lib.oracle_scores.argtypes = [vp, vp, i32, i32, i32, i32, i64, vp]
        lib.oracle_scores.restype = i32
        lib.oracle_topk_attention.argtypes = [vp, vp, vp, i32, i32, i32, i32, i64, i64,
                                              vp, vp, vp, vp]
        lib.oracle_topk_attention.restype = i32
        lib.oracle_topk_attention_window.argtypes = [vp, vp, vp, i32, i32, i32, i32, i64, i64, i64,
                                                     vp, vp, vp, vp]
        lib.oracle_topk_attention_window.restype = i32
        lib.oracle_topk_attention_multi.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i64, i32, i64, i64,
                                                    vp, vp, vp, vp]
        lib.oracle_topk_attention_multi.restype = i32
        lib.oracle_num_threads.restype = i32
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _check(a: np.ndarray, dtype: int) -> np.ndarray:
    want = {F32: np.float32, F16: np.float16, BF16: np.uint16}[dtype]
    if a.dtype != want:
        raise TypeError(f"expected {want} storage array for dtype code {dtype}, got {a.dtype}")
    return np.ascontiguousarray(a)


def scores(q: np.ndarray, K: np.ndarray, dtype: int) -> np.ndarray:
    """q [Hq,d], K [Hkv,N,d] storage arrays -> S [Hq,N] float64."""
    q, K = _check(q, dtype), _check(K, dtype)
    Hq, d = q.shape
    Hkv, N, _ = K.shape
    S = np.empty((Hq, N), dtype=np.float64)
    rc = _load().oracle_scores(q.ctypes.data, K.ctypes.data, dtype, Hq, Hkv, d, N, S.ctypes.data)
    if rc:
        raise RuntimeError(f"oracle_scores failed rc={rc}")
    return S


def topk_attention(q: np.ndarray, K: np.ndarray, V: np.ndarray, dtype: int, k: int):
    """Storage arrays in, (out [Hq,d] f64, idx [Hq,k] i64, vals [Hq,k] f64, lse [Hq] f64)."""
    q, K, V = _check(q, dtype), _check(K, dtype), _check(V, dtype)
    Hq, d = q.shape
    Hkv, N, _ = K.shape
    assert V.shape == K.shape
    out = np.empty((Hq, d), dtype=np.float64)
    idx = np.empty((Hq, k), dtype=np.int64)
    vals = np.empty((Hq, k), dtype=np.float64)
    lse = np.empty((Hq,), dtype=np.float64)
    rc = _load().oracle_topk_attention(q.ctypes.data, K.ctypes.data, V.ctypes.data, dtype,
                                       Hq, Hkv, d, N, k, out.ctypes.data, idx.ctypes.data,
                                       vals.ctypes.data, lse.ctypes.data)
    if rc:
        raise RuntimeError(f"oracle_topk_attention failed rc={rc}")
    return out, idx, vals, lse


def topk_attention_window(q: np.ndarray, K: np.ndarray, V: np.ndarray, dtype: int, k: int, window: int):
    """Like topk_attention, with the last `window` tokens always attended and the search
    restricted to the older prefix (one softmax over both parts)."""
    q, K, V = _check(q, dtype), _check(K, dtype), _check(V, dtype)
    Hq, d = q.shape
    Hkv, N, _ = K.shape
    out = np.empty((Hq, d), dtype=np.float64)
    idx = np.empty((Hq, k), dtype=np.int64)
    vals = np.empty((Hq, k), dtype=np.float64)
    lse = np.empty((Hq,), dtype=np.float64)
    rc = _load().oracle_topk_attention_window(q.ctypes.data, K.ctypes.data, V.ctypes.data, dtype,
                                              Hq, Hkv, d, N, k, window, out.ctypes.data, idx.ctypes.data,
                                              vals.ctypes.data, lse.ctypes.data)
    if rc:
        raise RuntimeError(f"oracle_topk_attention_window failed rc={rc}")
    return out, idx, vals, lse


def topk_attention_multi(q: np.ndarray, K: np.ndarray, V: np.ndarray, dtype: int, k: int, causal: bool,
                         window: int = 0):
    """q [M,Hq,d]: M queries against one cache, each an independent decode step; with `causal`
    query m sees the first N - (M - 1 - m) tokens.  Returns out [M,Hq,d], idx, vals [M,Hq,k], lse [M,Hq]."""
    q, K, V = _check(q, dtype), _check(K, dtype), _check(V, dtype)
    M, Hq, d = q.shape
    Hkv, N, _ = K.shape
    out = np.empty((M, Hq, d), dtype=np.float64)
    idx = np.empty((M, Hq, k), dtype=np.int64)
    vals = np.empty((M, Hq, k), dtype=np.float64)
    lse = np.empty((M, Hq), dtype=np.float64)
    rc = _load().oracle_topk_attention_multi(q.ctypes.data, K.ctypes.data, V.ctypes.data, dtype, M, Hq, Hkv, d,
                                             N, 1 if causal else 0, k, window, out.ctypes.data,
                                             idx.ctypes.data, vals.ctypes.data, lse.ctypes.data)
    if rc:
        raise RuntimeError(f"oracle_topk_attention_multi failed rc={rc}")
    return out, idx, vals, lse

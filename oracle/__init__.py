"""fp64 CPU oracle for packed variable-length causal attention (test infrastructure).

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import
this package; the GPU library never does.  The arithmetic lives in
``attn_oracle.c``; this file only marshals numpy arrays into it.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import numpy as np

from .build import LIBRARY, build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = build(force=False)
        lib = ctypes.CDLL(path)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        lib.oracle_attn_fwd.restype = ctypes.c_int
        lib.oracle_attn_fwd.argtypes = [dp, dp, dp, ip, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                        ctypes.c_int32, ctypes.c_double, dp, dp, dp]
        lib.oracle_attn_bwd.restype = ctypes.c_int
        lib.oracle_attn_bwd.argtypes = [dp, dp, dp, dp, ip, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                        ctypes.c_int32, ctypes.c_double, dp, dp, dp]
        lib.oracle_attn_rows.restype = ctypes.c_int
        lib.oracle_attn_rows.argtypes = [dp, dp, dp, dp, ip, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                         ctypes.c_int32, ctypes.c_double, ctypes.c_int32, ip, ip, dp, dp, dp]
        lib.oracle_attn_keys.restype = ctypes.c_int
        lib.oracle_attn_keys.argtypes = [dp, dp, dp, dp, ip, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                         ctypes.c_int32, ctypes.c_double, ctypes.c_int32, ip, ip, dp, dp]
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _dptr(a: Optional[np.ndarray]):
    if a is None:
        return None
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _as_f64(a: np.ndarray, shape: Tuple[int, ...]) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float64)
    if a.shape != shape:
        raise ValueError(f"expected shape {shape}, got {a.shape}")
    return a


def _cu(lengths: Sequence[int]) -> np.ndarray:
    cu = np.zeros(len(lengths) + 1, dtype=np.int32)
    np.cumsum(np.asarray(lengths, dtype=np.int64), out=cu[1:])
    return cu


def attn_fwd(q: np.ndarray, k: np.ndarray, v: np.ndarray, lengths: Sequence[int], scale: float,
             return_probs: bool = False):
    """q [T,Hq,d], k/v [T,Hkv,d] (any float dtype; converted exactly to fp64).

    Returns ``(o [T,Hq,d], lse [Hq,T])`` in fp64, plus ``probs [Hq,L,L]`` when
    ``return_probs`` (single-sequence packs only)."""
    lib = _load()
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    q = _as_f64(q, (T, Hq, d)); k = _as_f64(k, (T, Hkv, d)); v = _as_f64(v, (T, Hkv, d))
    cu = _cu(lengths)
    if int(cu[-1]) != T:
        raise ValueError("lengths do not sum to the token count")
    o = np.empty((T, Hq, d), dtype=np.float64)
    lse = np.empty((Hq, T), dtype=np.float64)
    probs = None
    if return_probs:
        if len(lengths) != 1:
            raise ValueError("probs only for a single sequence")
        probs = np.empty((Hq, T, T), dtype=np.float64)
    rc = lib.oracle_attn_fwd(_dptr(q), _dptr(k), _dptr(v), cu.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                             len(lengths), Hq, Hkv, d, float(scale), _dptr(o), _dptr(lse), _dptr(probs))
    if rc != 0:
        raise RuntimeError(f"oracle_attn_fwd failed with status {rc}")
    return (o, lse, probs) if return_probs else (o, lse)


def attn_bwd(q: np.ndarray, k: np.ndarray, v: np.ndarray, d_o: np.ndarray, lengths: Sequence[int],
             scale: float):
    """Returns ``(dq [T,Hq,d], dk [T,Hkv,d], dv [T,Hkv,d])`` in fp64."""
    lib = _load()
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    q = _as_f64(q, (T, Hq, d)); k = _as_f64(k, (T, Hkv, d)); v = _as_f64(v, (T, Hkv, d))
    d_o = _as_f64(d_o, (T, Hq, d))
    cu = _cu(lengths)
    if int(cu[-1]) != T:
        raise ValueError("lengths do not sum to the token count")
    dq = np.empty((T, Hq, d), dtype=np.float64)
    dk = np.empty((T, Hkv, d), dtype=np.float64)
    dv = np.empty((T, Hkv, d), dtype=np.float64)
    rc = lib.oracle_attn_bwd(_dptr(q), _dptr(k), _dptr(v), _dptr(d_o),
                             cu.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                             len(lengths), Hq, Hkv, d, float(scale), _dptr(dq), _dptr(dk), _dptr(dv))
    if rc != 0:
        raise RuntimeError(f"oracle_attn_bwd failed with status {rc}")
    return dq, dk, dv


def _iptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def attn_rows(q, k, v, d_o, lengths: Sequence[int], scale: float, tokens: Sequence[int], heads: Sequence[int]):
    """Sampled query rows: for each (packed token, q head) pair returns
    ``(o [n,d], lse [n], dq [n,d])`` without evaluating the other rows."""
    lib = _load()
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    q = _as_f64(q, (T, Hq, d)); k = _as_f64(k, (T, Hkv, d)); v = _as_f64(v, (T, Hkv, d))
    d_o = _as_f64(d_o, (T, Hq, d))
    cu = _cu(lengths)
    tok = np.ascontiguousarray(tokens, dtype=np.int32); hd = np.ascontiguousarray(heads, dtype=np.int32)
    n = len(tok)
    o = np.empty((n, d)); lse = np.empty(n); dq = np.empty((n, d))
    rc = lib.oracle_attn_rows(_dptr(q), _dptr(k), _dptr(v), _dptr(d_o), _iptr(cu), len(lengths), Hq, Hkv, d,
                              float(scale), n, _iptr(tok), _iptr(hd), _dptr(o), _dptr(lse), _dptr(dq))
    if rc != 0:
        raise RuntimeError(f"oracle_attn_rows failed with status {rc}")
    return o, lse, dq


def attn_keys(q, k, v, d_o, lengths: Sequence[int], scale: float, tokens: Sequence[int], kv_heads: Sequence[int]):
    """Sampled keys: for each (packed token, kv head) pair returns ``(dk [n,d], dv [n,d])``."""
    lib = _load()
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    q = _as_f64(q, (T, Hq, d)); k = _as_f64(k, (T, Hkv, d)); v = _as_f64(v, (T, Hkv, d))
    d_o = _as_f64(d_o, (T, Hq, d))
    cu = _cu(lengths)
    tok = np.ascontiguousarray(tokens, dtype=np.int32); hd = np.ascontiguousarray(kv_heads, dtype=np.int32)
    n = len(tok)
    dk = np.empty((n, d)); dv = np.empty((n, d))
    rc = lib.oracle_attn_keys(_dptr(q), _dptr(k), _dptr(v), _dptr(d_o), _iptr(cu), len(lengths), Hq, Hkv, d,
                              float(scale), n, _iptr(tok), _iptr(hd), _dptr(dk), _dptr(dv))
    if rc != 0:
        raise RuntimeError(f"oracle_attn_keys failed with status {rc}")
    return dk, dv

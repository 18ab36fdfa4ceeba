"""ctypes binding for the plain-C fp64 oracle in hydra_oracle.c (test infrastructure only).

The C file restates the same definition as reference.py with explicit loops; it exists so the
oracle can be evaluated (and timed as the CPU baseline) at the benchmark's full sizes.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hydra_oracle.c")
_LIB = os.path.join(_HERE, "libhydra_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile hydra_oracle.c with gcc (-O2, OpenMP).  Not tuned beyond that on purpose."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", _SRC, "-o", _LIB, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        lib.hydra_oracle_attn_varlen.restype = ctypes.c_int
        lib.hydra_oracle_attn_varlen.argtypes = [dp, dp, dp, dp, ip] + [ctypes.c_int] * 5 + [ctypes.c_double, ctypes.c_int,
                                                                                             ctypes.POINTER(ctypes.c_int)]
        lib.hydra_oracle_attn_rows.restype = ctypes.c_int
        lib.hydra_oracle_attn_rows.argtypes = [dp, dp, dp, ip] + [ctypes.c_int] * 5 + [ctypes.c_double, ip, ctypes.c_int, dp, dp,
                                                                                        ctypes.c_int]
        lib.hydra_oracle_unmasked_pairs.restype = ctypes.c_longlong
        lib.hydra_oracle_unmasked_pairs.argtypes = [ip, ctypes.c_int, ctypes.c_int]
        _lib = lib
    return _lib


def _d(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _i(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def attn_varlen(q, k, v, cu_seqlens, causal: bool, scale: float, nthreads: int = 0, return_threads: bool = False):
    lib = _load()
    q = np.ascontiguousarray(q, dtype=np.float64)
    k = np.ascontiguousarray(k, dtype=np.float64)
    v = np.ascontiguousarray(v, dtype=np.float64)
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    N, Hq, d = q.shape
    Hkv = k.shape[1]
    if cu[0] != 0 or cu[-1] != N or k.shape != v.shape or k.shape[0] != N or k.shape[2] != d:
        raise ValueError("inconsistent shapes")
    out = np.zeros_like(q)
    used = ctypes.c_int(0)
    rc = lib.hydra_oracle_attn_varlen(_d(q), _d(k), _d(v), _d(out), _i(cu), len(cu) - 1, Hq, Hkv, d, int(bool(causal)),
                                      float(scale), int(nthreads), ctypes.byref(used))
    if rc != 0:
        raise RuntimeError(f"hydra_oracle_attn_varlen failed with {rc}")
    return (out, used.value) if return_threads else out


def attn_rows(q, k, v, cu_seqlens, causal: bool, scale: float, rows, return_probs: bool = False):
    lib = _load()
    q = np.ascontiguousarray(q, dtype=np.float64)
    k = np.ascontiguousarray(k, dtype=np.float64)
    v = np.ascontiguousarray(v, dtype=np.float64)
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    rows = np.ascontiguousarray(np.asarray(list(rows), dtype=np.int32).reshape(-1, 2))
    N, Hq, d = q.shape
    out = np.zeros((rows.shape[0], d), dtype=np.float64)
    max_len = int(np.diff(cu).max()) if len(cu) > 1 else 0
    probs = np.zeros((rows.shape[0], max_len), dtype=np.float64) if return_probs else None
    rc = lib.hydra_oracle_attn_rows(_d(q), _d(k), _d(v), _i(cu), len(cu) - 1, Hq, k.shape[1], d, int(bool(causal)), float(scale),
                                    _i(rows), rows.shape[0], _d(out), _d(probs) if return_probs else None, max_len)
    if rc != 0:
        raise RuntimeError(f"hydra_oracle_attn_rows failed with {rc}")
    return (out, probs) if return_probs else out


def unmasked_pairs(cu_seqlens, causal: bool) -> int:
    lib = _load()
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    return int(lib.hydra_oracle_unmasked_pairs(_i(cu), len(cu) - 1, int(bool(causal))))

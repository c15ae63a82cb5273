"""ctypes front for the C oracle (oracle/pods_oracle.c).  TEST INFRASTRUCTURE ONLY.

Compiles the C file with gcc on first use if no built library is present.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pods_oracle.c")
_LIB = os.path.join(_HERE, "libpods_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_select.restype = ctypes.c_int
        _lib.oracle_advantage.restype = ctypes.c_int
    return _lib


def select(rewards: np.ndarray, m: int, threads: int = 0):
    """Batched Alg. 2 -> (sel_idx[B, m] int32, sel_k[B] int32, threads_used)."""
    lib = _load()
    r = np.ascontiguousarray(rewards, dtype=np.float32)
    B, n = r.shape
    idx = np.empty((B, m), dtype=np.int32)
    ks = np.empty(B, dtype=np.int32)
    rc = lib.oracle_select(r.ctypes.data_as(ctypes.c_void_p), ctypes.c_int32(B), ctypes.c_int32(n),
                           ctypes.c_int32(m), idx.ctypes.data_as(ctypes.c_void_p),
                           ks.ctypes.data_as(ctypes.c_void_p), ctypes.c_int32(threads))
    if rc >= 0:
        raise ValueError("oracle_select rejected its arguments")
    return idx, ks, -rc


def advantage(rewards: np.ndarray, sel_idx: np.ndarray, std_eps: float = 0.0) -> np.ndarray:
    lib = _load()
    r = np.ascontiguousarray(rewards, dtype=np.float32)
    s = np.ascontiguousarray(sel_idx, dtype=np.int32)
    B, n = r.shape
    m = s.shape[1]
    out = np.empty((B, m), dtype=np.float64)
    rc = lib.oracle_advantage(r.ctypes.data_as(ctypes.c_void_p), s.ctypes.data_as(ctypes.c_void_p),
                              ctypes.c_int32(B), ctypes.c_int32(n), ctypes.c_int32(m),
                              ctypes.c_double(std_eps), out.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise ValueError("oracle_advantage rejected its arguments")
    return out

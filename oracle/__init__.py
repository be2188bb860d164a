"""CPU oracle of the fixed-routing MoE expert layer - TEST INFRASTRUCTURE ONLY.

Importable by the tests, the smoke check and the benchmark's ``cpu_baseline`` leg; never by the
product package.  It wraps ``oracle/grouter_oracle.c`` (plain C loops that evaluate Eq. 1 of Sec. 2.1
token by token, the App. A expert gradient, and a textbook stable counting sort) through ctypes, and
shares nothing with the HIP path.  Everything here works on host numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_SRC = [os.path.join(_HERE, "grouter_oracle.c"), os.path.join(_HERE, "moe_body.inc")]
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O3, OpenMP, baseline x86-64 so the library runs on any host) into oracle/liboracle.so."""
    stale = (not os.path.exists(_SO)) or any(os.path.getmtime(s) > os.path.getmtime(_SO) for s in _SRC)
    if force or stale:
        cmd = ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra", "-o", _SO, _SRC[0], "-lm"]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _SO


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_SO)
        i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        lib.oracle_plan.argtypes = [vp, i64, i32, vp, vp, vp, vp]
        lib.oracle_plan.restype = ctypes.c_int
        lib.oracle_num_threads.restype = ctypes.c_int
        for sfx in ("f32", "f64"):
            fwd = getattr(lib, f"oracle_moe_fwd_{sfx}")
            fwd.argtypes = [i64, i32, i32, i32, i32] + [vp] * 7
            fwd.restype = None
            bwd = getattr(lib, f"oracle_moe_bwd_{sfx}")
            bwd.argtypes = [i64, i32, i32, i32, i32] + [vp] * 11
            bwd.restype = None
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32, exactly."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def plan(idx: np.ndarray, E: int):
    """Stable counting sort of the routed slots: (counts[E], offsets[E+1], row_to_src[N], src_to_row[N])."""
    flat = np.ascontiguousarray(idx, dtype=np.int32).reshape(-1)
    N = flat.size
    counts = np.zeros(E, dtype=np.int32)
    offsets = np.zeros(E + 1, dtype=np.int32)
    r2s = np.zeros(max(N, 1), dtype=np.int32)
    s2r = np.zeros(max(N, 1), dtype=np.int32)
    rc = _load().oracle_plan(_ptr(flat), N, E, _ptr(counts), _ptr(offsets), _ptr(r2s), _ptr(s2r))
    if rc != 0:
        raise ValueError("expert id outside [0, E)")
    return counts, offsets, r2s[:N], s2r[:N]


def _prep(dtype, x, w, idx, W1, W3, W2):
    x = np.ascontiguousarray(x, dtype=dtype)
    T, d = x.shape
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    k = idx.shape[1]
    w = np.ascontiguousarray(w, dtype=dtype).reshape(T, k)
    W1 = np.ascontiguousarray(W1, dtype=dtype)
    W3 = np.ascontiguousarray(W3, dtype=dtype)
    W2 = np.ascontiguousarray(W2, dtype=dtype)
    E, d1, f = W1.shape
    if not (d1 == d and W3.shape == (E, d, f) and W2.shape == (E, f, d) and idx.shape == (T, k)):
        raise ValueError("shape mismatch")
    if idx.size and (idx.min() < 0 or idx.max() >= E):
        raise ValueError("expert id outside [0, E)")
    return x, w, idx, W1, W3, W2, T, d, f, E, k


def moe_fwd(x, w, idx, W1, W3, W2, dtype=np.float64) -> np.ndarray:
    """y[T,d] of Eq. 1 under the given routing, in ``dtype`` (float64 or float32) arithmetic."""
    x, w, idx, W1, W3, W2, T, d, f, E, k = _prep(dtype, x, w, idx, W1, W3, W2)
    y = np.empty((T, d), dtype=dtype)
    fn = getattr(_load(), "oracle_moe_fwd_f64" if dtype == np.float64 else "oracle_moe_fwd_f32")
    fn(T, d, f, E, k, _ptr(x), _ptr(w), _ptr(idx), _ptr(W1), _ptr(W3), _ptr(W2), _ptr(y))
    return y


def moe_bwd(x, w, idx, W1, W3, W2, dY, dtype=np.float64):
    """(dX, dW1, dW3, dW2) of L = <y, dY> with the routing held fixed."""
    x, w, idx, W1, W3, W2, T, d, f, E, k = _prep(dtype, x, w, idx, W1, W3, W2)
    dY = np.ascontiguousarray(dY, dtype=dtype)
    if dY.shape != (T, d):
        raise ValueError("shape mismatch")
    dX = np.empty((T, d), dtype=dtype)
    dW1 = np.empty((E, d, f), dtype=dtype)
    dW3 = np.empty((E, d, f), dtype=dtype)
    dW2 = np.empty((E, f, d), dtype=dtype)
    fn = getattr(_load(), "oracle_moe_bwd_f64" if dtype == np.float64 else "oracle_moe_bwd_f32")
    fn(T, d, f, E, k, _ptr(x), _ptr(w), _ptr(idx), _ptr(W1), _ptr(W3), _ptr(W2), _ptr(dY), _ptr(dX), _ptr(dW1),
       _ptr(dW3), _ptr(dW2))
    return dX, dW1, dW3, dW2

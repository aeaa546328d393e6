"""ctypes front end of the CPU oracle (``attn_ref.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, ``__graft_entry__.smoke()``
and the ``cpu_baseline`` leg of ``bench.py``.  It imports nothing from the GPU
package and the GPU package imports nothing from here.

The arithmetic lives in ``attn_ref.c`` (fp64, plain definition of attention as
the paper's Section 3.4.2 stages T = QK^T, C = softmax, U = PV compose it);
this file only builds the shared object with gcc and marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attn_ref.c")
_LIB = os.path.join(_HERE, "libattn_ref.so")

FP16 = 0
BF16 = 1
E4M3 = 2     # OCP 8-bit float (1-4-3, bias 7, no infinities), stored as uint8

_lib = None


def build(force: bool = False) -> str:
    """Compile ``attn_ref.c`` into ``libattn_ref.so`` next to it (gcc, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        u16p = ctypes.c_void_p          # raw storage patterns: uint16 (fp16, bf16) or uint8 (E4M3)
        f64p = ctypes.POINTER(ctypes.c_double)
        i32p = ctypes.POINTER(ctypes.c_int)
        lib.attn_ref_f64.restype = ctypes.c_int
        lib.attn_ref_f64.argtypes = [u16p, u16p, u16p, ctypes.c_int, f64p, f64p, f64p,
                                     ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                     ctypes.c_double, ctypes.c_int, ctypes.c_int]
        lib.attn_ref_rows_f64.restype = ctypes.c_int
        lib.attn_ref_rows_f64.argtypes = [u16p, u16p, u16p, ctypes.c_int, i32p, ctypes.c_int,
                                          f64p, f64p, f64p,
                                          ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                          ctypes.c_double, ctypes.c_int, ctypes.c_int]
        lib.attn_ref_decode.restype = None
        lib.attn_ref_decode.argtypes = [u16p, f64p, ctypes.c_long, ctypes.c_int]
        lib.attn_ref_max_threads.restype = ctypes.c_int
        lib.attn_ref_max_threads.argtypes = []
        _lib = lib
    return _lib


def _storage(dtype: int):
    return np.uint8 if dtype == E4M3 else np.uint16


def _bits(a: np.ndarray, shape, dtype: int) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != _storage(dtype):
        raise TypeError("oracle inputs are raw %s bit patterns for dtype %d, got %s"
                        % (np.dtype(_storage(dtype)).name, dtype, a.dtype))
    if tuple(a.shape) != tuple(shape):
        raise ValueError("expected shape %s, got %s" % (shape, a.shape))
    return a


def _ptr(a: np.ndarray, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _raw(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def max_threads() -> int:
    """Threads the oracle uses when ``nthreads=0`` (OpenMP's default team size)."""
    return int(_load().attn_ref_max_threads())


def decode(bits: np.ndarray, dtype: int) -> np.ndarray:
    """Exact fp16/bf16/E4M3 bit pattern -> float64, by the oracle's own decoder."""
    bits = np.ascontiguousarray(bits, dtype=_storage(dtype))
    out = np.empty(bits.shape, dtype=np.float64)
    _load().attn_ref_decode(_raw(bits), _ptr(out, ctypes.c_double), bits.size, dtype)
    return out


def attn_ref(q, k, v, dtype: int, scale: float, causal: bool, nthreads: int = 0, return_p: bool = False):
    """Full attention forward of ``[B,H,N,d]`` tensors of raw bit patterns (uint16, or uint8 for E4M3).

    Returns ``(O [B,H,N,d] f64, LSE [B,H,N] f64)`` and, with ``return_p``, the
    normalised probability matrices ``[B,H,N,N]``.
    """
    B, H, N, d = q.shape
    q = _bits(q, (B, H, N, d), dtype); k = _bits(k, (B, H, N, d), dtype); v = _bits(v, (B, H, N, d), dtype)
    o = np.empty((B, H, N, d), dtype=np.float64)
    lse = np.empty((B, H, N), dtype=np.float64)
    p = np.empty((B, H, N, N), dtype=np.float64) if return_p else None
    rc = _load().attn_ref_f64(_raw(q), _raw(k), _raw(v),
                              dtype, _ptr(o, ctypes.c_double), _ptr(lse, ctypes.c_double),
                              _ptr(p, ctypes.c_double) if return_p else None,
                              B, H, N, d, float(scale), int(bool(causal)), int(nthreads))
    if rc != 0:
        raise RuntimeError("attn_ref_f64 failed with code %d" % rc)
    return (o, lse, p) if return_p else (o, lse)


def attn_ref_rows(q, k, v, dtype: int, rows, scale: float, causal: bool, nthreads: int = 0,
                  return_p: bool = False):
    """The same definition for sampled query rows ``rows = [(b, h, i), ...]``.

    Returns ``(O_rows [n,d] f64, LSE_rows [n] f64)`` and, with ``return_p``, the
    rows' normalised probabilities ``[n,N]``.
    """
    B, H, N, d = q.shape
    q = _bits(q, (B, H, N, d), dtype); k = _bits(k, (B, H, N, d), dtype); v = _bits(v, (B, H, N, d), dtype)
    rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int32).reshape(-1, 3))
    n = rows.shape[0]
    o = np.empty((n, d), dtype=np.float64)
    lse = np.empty((n,), dtype=np.float64)
    p = np.empty((n, N), dtype=np.float64) if return_p else None
    rc = _load().attn_ref_rows_f64(_raw(q), _raw(k), _raw(v),
                                   dtype, _ptr(rows, ctypes.c_int), n,
                                   _ptr(o, ctypes.c_double), _ptr(lse, ctypes.c_double),
                                   _ptr(p, ctypes.c_double) if return_p else None,
                                   B, H, N, d, float(scale), int(bool(causal)), int(nthreads))
    if rc != 0:
        raise RuntimeError("attn_ref_rows_f64 failed with code %d" % rc)
    return (o, lse, p) if return_p else (o, lse)

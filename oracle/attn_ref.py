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
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f64p = ctypes.POINTER(ctypes.c_double)
        i32p = ctypes.POINTER(ctypes.c_int)
        lib.attn_ref_f64.restype = ctypes.c_int
        lib.attn_ref_f64.argtypes = [u16p, u16p, u16p, ctypes.c_int, f64p, f64p, f64p,
                                     ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                     ctypes.c_double, ctypes.c_int, ctypes.c_int]
        lib.attn_ref_rows_f64.restype = ctypes.c_int
        lib.attn_ref_rows_f64.argtypes = [u16p, u16p, u16p, ctypes.c_int, i32p, ctypes.c_int,
                                          f64p, f64p,
                                          ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                          ctypes.c_double, ctypes.c_int, ctypes.c_int]
        lib.attn_ref_decode.restype = None
        lib.attn_ref_decode.argtypes = [u16p, f64p, ctypes.c_long, ctypes.c_int]
        lib.attn_ref_max_threads.restype = ctypes.c_int
        lib.attn_ref_max_threads.argtypes = []
        _lib = lib
    return _lib


def _u16(a: np.ndarray, shape) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("oracle inputs are raw uint16 bit patterns, got %s" % a.dtype)
    if tuple(a.shape) != tuple(shape):
        raise ValueError("expected shape %s, got %s" % (shape, a.shape))
    return a


def _ptr(a: np.ndarray, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def max_threads() -> int:
    """Threads the oracle uses when ``nthreads=0`` (OpenMP's default team size)."""
    return int(_load().attn_ref_max_threads())


def decode(bits: np.ndarray, dtype: int) -> np.ndarray:
    """Exact fp16/bf16 bit pattern -> float64, by the oracle's own decoder."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, dtype=np.float64)
    _load().attn_ref_decode(_ptr(bits, ctypes.c_uint16), _ptr(out, ctypes.c_double), bits.size, dtype)
    return out


def attn_ref(q, k, v, dtype: int, scale: float, causal: bool, nthreads: int = 0, return_p: bool = False):
    """Full attention forward of ``[B,H,N,d]`` uint16 tensors.

    Returns ``(O [B,H,N,d] f64, LSE [B,H,N] f64)`` and, with ``return_p``, the
    normalised probability matrices ``[B,H,N,N]``.
    """
    B, H, N, d = q.shape
    q = _u16(q, (B, H, N, d)); k = _u16(k, (B, H, N, d)); v = _u16(v, (B, H, N, d))
    o = np.empty((B, H, N, d), dtype=np.float64)
    lse = np.empty((B, H, N), dtype=np.float64)
    p = np.empty((B, H, N, N), dtype=np.float64) if return_p else None
    rc = _load().attn_ref_f64(_ptr(q, ctypes.c_uint16), _ptr(k, ctypes.c_uint16), _ptr(v, ctypes.c_uint16),
                              dtype, _ptr(o, ctypes.c_double), _ptr(lse, ctypes.c_double),
                              _ptr(p, ctypes.c_double) if return_p else None,
                              B, H, N, d, float(scale), int(bool(causal)), int(nthreads))
    if rc != 0:
        raise RuntimeError("attn_ref_f64 failed with code %d" % rc)
    return (o, lse, p) if return_p else (o, lse)


def attn_ref_rows(q, k, v, dtype: int, rows, scale: float, causal: bool, nthreads: int = 0):
    """The same definition for sampled query rows ``rows = [(b, h, i), ...]``.

    Returns ``(O_rows [n,d] f64, LSE_rows [n] f64)``.
    """
    B, H, N, d = q.shape
    q = _u16(q, (B, H, N, d)); k = _u16(k, (B, H, N, d)); v = _u16(v, (B, H, N, d))
    rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int32).reshape(-1, 3))
    n = rows.shape[0]
    o = np.empty((n, d), dtype=np.float64)
    lse = np.empty((n,), dtype=np.float64)
    rc = _load().attn_ref_rows_f64(_ptr(q, ctypes.c_uint16), _ptr(k, ctypes.c_uint16), _ptr(v, ctypes.c_uint16),
                                   dtype, _ptr(rows, ctypes.c_int), n,
                                   _ptr(o, ctypes.c_double), _ptr(lse, ctypes.c_double),
                                   B, H, N, d, float(scale), int(bool(causal)), int(nthreads))
    if rc != 0:
        raise RuntimeError("attn_ref_rows_f64 failed with code %d" % rc)
    return o, lse

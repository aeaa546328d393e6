"""ctypes front end of the CPU oracle of the NT matrix product (``gemm_ref.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, ``__graft_entry__.smoke()``
and the ``cpu_baseline`` leg of ``bench.py``.  It imports nothing from the GPU
package and the GPU package imports nothing from here.

The arithmetic lives in ``gemm_ref.c`` (fp64, the plain definition
``C[m][n] = sum_k A[m][k] * B[n][k]`` of the product the paper's Section 3.1
program accumulates and Section 5.2 benchmarks); this file only builds the
shared object with gcc and marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gemm_ref.c")
_LIB = os.path.join(_HERE, "libgemm_ref.so")

FP16 = 0
BF16 = 1
E4M3 = 2     # OCP 8-bit float, stored as uint8

_lib = None


def build(force: bool = False) -> str:
    """Compile ``gemm_ref.c`` into ``libgemm_ref.so`` next to it (gcc, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                        "-o", tmp, _SRC, "-lm"], check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        f64p, i32p = (ctypes.POINTER(t) for t in (ctypes.c_double, ctypes.c_int))
        u16p = ctypes.c_void_p          # raw storage patterns: uint16 (fp16, bf16) or uint8 (E4M3)
        ci = ctypes.c_int
        lib.gemm_ref_nt_f64.restype = ci
        lib.gemm_ref_nt_f64.argtypes = [u16p, u16p, ci, f64p, ci, ci, ci, ci]
        lib.gemm_ref_nt_samples_f64.restype = ci
        lib.gemm_ref_nt_samples_f64.argtypes = [u16p, u16p, ci, i32p, ci, f64p, ci, ci, ci]
        lib.gemm_ref_decode.restype = None
        lib.gemm_ref_decode.argtypes = [u16p, f64p, ctypes.c_long, ci]
        lib.gemm_ref_max_threads.restype = ci
        lib.gemm_ref_max_threads.argtypes = []
        _lib = lib
    return _lib


def _storage(dtype: int):
    return np.uint8 if dtype == E4M3 else np.uint16


def _bits(a, shape, dtype: int):
    a = np.ascontiguousarray(a)
    if a.dtype != _storage(dtype):
        raise TypeError("oracle inputs are raw %s bit patterns for dtype %d, got %s"
                        % (np.dtype(_storage(dtype)).name, dtype, a.dtype))
    if tuple(a.shape) != tuple(shape):
        raise ValueError("expected shape %s, got %s" % (shape, a.shape))
    return a


def _raw(a):
    return ctypes.c_void_p(a.ctypes.data)


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def max_threads() -> int:
    return int(_load().gemm_ref_max_threads())


def decode(bits, dtype: int) -> np.ndarray:
    """Exact fp16/bf16/E4M3 bit pattern -> float64, by the oracle's own decoder."""
    bits = np.ascontiguousarray(bits, dtype=_storage(dtype))
    out = np.empty(bits.shape, dtype=np.float64)
    _load().gemm_ref_decode(_raw(bits), _ptr(out, ctypes.c_double), bits.size, dtype)
    return out


def gemm_nt(a, b, dtype: int, nthreads: int = 0) -> np.ndarray:
    """``C = A B^T`` in fp64 for ``a`` [M,K] and ``b`` [N,K] bit patterns (uint16, or uint8 for E4M3); returns [M,N] float64."""
    M, K = a.shape
    N = b.shape[0]
    a = _bits(a, (M, K), dtype); b = _bits(b, (N, K), dtype)
    c = np.empty((M, N), dtype=np.float64)
    rc = _load().gemm_ref_nt_f64(_raw(a), _raw(b), dtype, _ptr(c, ctypes.c_double),
                                 M, N, K, int(nthreads))
    if rc != 0:
        raise RuntimeError("gemm_ref_nt_f64 failed with code %d" % rc)
    return c


def gemm_nt_samples(a, b, dtype: int, idx) -> np.ndarray:
    """The same definition for sampled entries ``idx = [(m, n), ...]``; returns [len(idx)] float64."""
    M, K = a.shape
    N = b.shape[0]
    a = _bits(a, (M, K), dtype); b = _bits(b, (N, K), dtype)
    idx = np.ascontiguousarray(np.asarray(idx, dtype=np.int32).reshape(-1, 2))
    out = np.empty((idx.shape[0],), dtype=np.float64)
    rc = _load().gemm_ref_nt_samples_f64(_raw(a), _raw(b), dtype,
                                         _ptr(idx, ctypes.c_int), idx.shape[0], _ptr(out, ctypes.c_double), M, N, K)
    if rc != 0:
        raise RuntimeError("gemm_ref_nt_samples_f64 failed with code %d" % rc)
    return out

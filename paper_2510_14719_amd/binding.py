"""Thin ctypes binding of ``libattn_fwd.so`` (the C ABI of ``include/attn_fwd.h``).

Argument marshalling only: every step of the attention forward pass runs in the
HIP kernels behind the C ABI.  Torch tensors are accepted for their device
memory (``data_ptr()``) and the current stream handle; nothing is computed in
Python and there is no fallback: without the built library, or without a GPU
for the tensors, the calls raise.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libattn_fwd.so")

FP16 = 0
BF16 = 1

_lib = None


class AttnFwdError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("attn_fwd failed with code %d: %s" % (code, text))
        self.code = code


def load_library() -> ctypes.CDLL:
    """Load the in-tree shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "%s is missing: build it with `python -m paper_2510_14719_amd.build` "
                "(there is no CPU fallback)" % LIB_PATH)
        # PyTorch provides the device memory and the streams, so its HIP runtime must be the one
        # this process uses: load it first, and the library's libamdhip64 dependency resolves to
        # the copy torch has already mapped instead of a second runtime with its own streams.
        import torch  # noqa: F401
        lib = ctypes.CDLL(LIB_PATH)
        vp, fp, ci, cf = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_float
        common = [vp, vp, vp, vp, fp, ci, ci, ci, ci, cf, ci, vp]
        lib.attn_fwd_f16.restype = ci
        lib.attn_fwd_f16.argtypes = common
        lib.attn_fwd_bf16.restype = ci
        lib.attn_fwd_bf16.argtypes = common
        lib.attn_fwd.restype = ci
        lib.attn_fwd.argtypes = common + [ci]
        lib.attn_fwd_check_args.restype = ci
        lib.attn_fwd_check_args.argtypes = [vp, vp, vp, vp, fp, ci, ci, ci, ci, cf, ci]
        lib.attn_fwd_fp8.restype = ci
        lib.attn_fwd_fp8.argtypes = common + [ci]
        lib.attn_fwd_fp8_check_args.restype = ci
        lib.attn_fwd_fp8_check_args.argtypes = [vp, vp, vp, vp, fp, ci, ci, ci, ci, cf, ci]
        lib.attn_fwd_fp8_tile_param.restype = ci
        lib.attn_fwd_fp8_tile_param.argtypes = [ci, ci]
        lib.attn_fwd_strerror.restype = ctypes.c_char_p
        lib.attn_fwd_strerror.argtypes = [ci]
        lib.attn_fwd_version.restype = ci
        lib.attn_fwd_version.argtypes = []
        lib.attn_fwd_tile_param.restype = ci
        lib.attn_fwd_tile_param.argtypes = [ci, ci, ci]
        lib.attn_fwd_tile_schedule.restype = ci
        lib.attn_fwd_tile_schedule.argtypes = [ci, ci, ci, ci]
        lib.attn_fwd_mfma_probe.restype = ci
        lib.attn_fwd_mfma_probe.argtypes = [vp, ci, ci, ci, ci, vp]
        lib.attn_fwd_mfma_probe_flops.restype = ctypes.c_double
        lib.attn_fwd_mfma_probe_flops.argtypes = [ci, ci]
        lib.attn_fwd_mfma_probe_flops_of.restype = ctypes.c_double
        lib.attn_fwd_mfma_probe_flops_of.argtypes = [ci, ci, ci]
        lib.attn_fwd_mfma_probe_sink_floats.restype = ci
        lib.attn_fwd_mfma_probe_sink_floats.argtypes = [ci]
        lib.gemm_nt.restype = ci
        lib.gemm_nt.argtypes = [vp, vp, vp, ci, ci, ci, vp, ci]
        lib.gemm_nt_config.restype = ci
        lib.gemm_nt_config.argtypes = [vp, vp, vp, ci, ci, ci, vp, ci, ci]
        lib.gemm_nt_f16.restype = ci
        lib.gemm_nt_f16.argtypes = [vp, vp, vp, ci, ci, ci, vp]
        lib.gemm_nt_bf16.restype = ci
        lib.gemm_nt_bf16.argtypes = [vp, vp, vp, ci, ci, ci, vp]
        lib.gemm_nt_check_args.restype = ci
        lib.gemm_nt_check_args.argtypes = [vp, vp, vp, ci, ci, ci, ci]
        lib.gemm_nt_strerror.restype = ctypes.c_char_p
        lib.gemm_nt_strerror.argtypes = [ci]
        lib.gemm_nt_tile_param.restype = ci
        lib.gemm_nt_tile_param.argtypes = [ci]
        lib.gemm_nt_fp8.restype = ci
        lib.gemm_nt_fp8.argtypes = [vp, vp, vp, ci, ci, ci, vp, ci]
        lib.gemm_nt_fp8_config.restype = ci
        lib.gemm_nt_fp8_config.argtypes = [vp, vp, vp, ci, ci, ci, vp, ci, ci]
        lib.gemm_nt_fp8_check_args.restype = ci
        lib.gemm_nt_fp8_check_args.argtypes = [vp, vp, vp, ci, ci, ci, ci]
        lib.gemm_nt_fp8_tile_param.restype = ci
        lib.gemm_nt_fp8_tile_param.argtypes = [ci]
        _lib = lib
    return _lib


def strerror(code: int) -> str:
    return load_library().attn_fwd_strerror(int(code)).decode()


def _ptr(x) -> int:
    """Device address of a torch tensor, or an integer address passed through."""
    if isinstance(x, int):
        return x
    if not x.is_cuda:
        raise ValueError("attn_fwd takes device tensors; got a tensor on %s" % x.device)
    if not x.is_contiguous():
        raise ValueError("attn_fwd takes contiguous [B,H,N,d] tensors")
    return x.data_ptr()


def _stream_handle(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def attn_fwd_raw(q, k, v, o, lse, B, H, N, d, scale, causal, stream, dtype) -> int:
    """The C call itself; returns its code without raising."""
    return int(load_library().attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), int(B), int(H), int(N), int(d),
                                       float(scale), int(bool(causal)), _stream_handle(stream), int(dtype)))


def attn_fwd(q, k, v, o, lse, B, H, N, d, scale, causal, stream=None, dtype=None) -> None:
    """``attn_fwd(q, k, v, o, lse, B, H, N, d, scale, causal, stream)`` of the C ABI.

    ``dtype`` defaults to the element type of ``q`` (float16 -> FP16, bfloat16 or
    a 16-bit integer view needs an explicit ``dtype``).  Asynchronous: the kernel
    is enqueued on ``stream`` (default: torch's current stream) and the call returns.
    """
    if dtype is None:
        import torch
        if q.dtype == torch.float16:
            dtype = FP16
        elif q.dtype == torch.bfloat16:
            dtype = BF16
        else:
            raise ValueError("pass dtype=FP16/BF16 for tensors of type %s" % q.dtype)
    rc = attn_fwd_raw(q, k, v, o, lse, B, H, N, d, scale, causal, stream, dtype)
    if rc != 0:
        raise AttnFwdError(rc, strerror(rc))


def attn_fwd_f16(q, k, v, o, lse, B, H, N, d, scale, causal, stream=None) -> None:
    rc = int(load_library().attn_fwd_f16(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), int(B), int(H), int(N), int(d),
                                         float(scale), int(bool(causal)), _stream_handle(stream)))
    if rc != 0:
        raise AttnFwdError(rc, strerror(rc))


def attn_fwd_bf16(q, k, v, o, lse, B, H, N, d, scale, causal, stream=None) -> None:
    rc = int(load_library().attn_fwd_bf16(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), int(B), int(H), int(N), int(d),
                                          float(scale), int(bool(causal)), _stream_handle(stream)))
    if rc != 0:
        raise AttnFwdError(rc, strerror(rc))


def attn_fwd_fp8_raw(q, k, v, o, lse, B, H, N, d, scale, causal, stream, out_dtype) -> int:
    """The C call itself; returns its code without raising."""
    return int(load_library().attn_fwd_fp8(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), int(B), int(H), int(N), int(d),
                                           float(scale), int(bool(causal)), _stream_handle(stream), int(out_dtype)))


def attn_fwd_fp8(q, k, v, o, lse, B, H, N, d, scale, causal, stream=None, out_dtype=None) -> None:
    """``attn_fwd_fp8`` of the C ABI: Q, K, V one byte per element (E4M3), O in fp16 or bf16.

    ``out_dtype`` defaults to the element type of ``o``.  Asynchronous, like ``attn_fwd``.
    """
    if out_dtype is None:
        import torch
        if o.dtype == torch.float16:
            out_dtype = FP16
        elif o.dtype == torch.bfloat16:
            out_dtype = BF16
        else:
            raise ValueError("pass out_dtype=FP16/BF16 for an output tensor of type %s" % o.dtype)
    rc = attn_fwd_fp8_raw(q, k, v, o, lse, B, H, N, d, scale, causal, stream, out_dtype)
    if rc != 0:
        raise AttnFwdError(rc, strerror(rc))


def fp8_tile_params(d: int) -> dict:
    lib = load_library()
    return {"BM": lib.attn_fwd_fp8_tile_param(d, 0), "BN": lib.attn_fwd_fp8_tile_param(d, 1),
            "stages": lib.attn_fwd_fp8_tile_param(d, 2), "threads": lib.attn_fwd_fp8_tile_param(d, 3)}


def tile_params(d: int, causal: bool = False) -> dict:
    lib = load_library()
    return {"BM": lib.attn_fwd_tile_param(d, int(causal), 0), "BN": lib.attn_fwd_tile_param(d, int(causal), 1),
            "stages": lib.attn_fwd_tile_param(d, int(causal), 2), "threads": lib.attn_fwd_tile_param(d, int(causal), 3)}


def mfma_probe(sink, workgroups: int, iters: int, random_operands: bool, dtype: int = FP16, stream=None) -> float:
    """``attn_fwd_mfma_probe`` of the C ABI: enqueue the register-only MFMA stream; returns its flop count."""
    lib = load_library()
    need = lib.attn_fwd_mfma_probe_sink_floats(int(workgroups))
    if not isinstance(sink, int) and sink.numel() * sink.element_size() < 4 * need:
        raise ValueError("sink needs %d floats" % need)
    rc = int(lib.attn_fwd_mfma_probe(_ptr(sink), int(workgroups), int(iters), int(bool(random_operands)), int(dtype),
                                     _stream_handle(stream)))
    if rc != 0:
        raise AttnFwdError(rc, strerror(rc))
    return float(lib.attn_fwd_mfma_probe_flops_of(int(workgroups), int(iters), int(dtype)))


class GemmNtError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("gemm_nt failed with code %d: %s" % (code, text))
        self.code = code


def gemm_nt_raw(a, b, c, M, N, K, stream, dtype, config=None) -> int:
    """The C call itself (``gemm_nt``, or ``gemm_nt_config`` when a configuration is given); returns its code
    without raising."""
    lib = load_library()
    if config is None:
        return int(lib.gemm_nt(_ptr(a), _ptr(b), _ptr(c), int(M), int(N), int(K), _stream_handle(stream), int(dtype)))
    return int(lib.gemm_nt_config(_ptr(a), _ptr(b), _ptr(c), int(M), int(N), int(K), _stream_handle(stream), int(dtype), int(config)))


def gemm_nt(a, b, c, M, N, K, stream=None, dtype=None, config=None) -> None:
    """``gemm_nt(a, b, c, M, N, K, stream, dtype)`` of the C ABI: ``C = A B^T`` for ``a`` [M,K], ``b`` [N,K].

    ``dtype`` defaults to the element type of ``a``.  Asynchronous: the kernel is enqueued on
    ``stream`` (default: torch's current stream) and the call returns.
    """
    if dtype is None:
        import torch
        if a.dtype == torch.float16:
            dtype = FP16
        elif a.dtype == torch.bfloat16:
            dtype = BF16
        else:
            raise ValueError("pass dtype=FP16/BF16 for tensors of type %s" % a.dtype)
    rc = gemm_nt_raw(a, b, c, M, N, K, stream, dtype, config)
    if rc != 0:
        raise GemmNtError(rc, load_library().gemm_nt_strerror(rc).decode())


def gemm_tile_params() -> dict:
    lib = load_library()
    return {"BM": lib.gemm_nt_tile_param(0), "BN": lib.gemm_nt_tile_param(1), "BK": lib.gemm_nt_tile_param(2),
            "stages": lib.gemm_nt_tile_param(3), "threads": lib.gemm_nt_tile_param(4)}


def gemm_nt_fp8_raw(a, b, c, M, N, K, stream, out_dtype, config=None) -> int:
    """The C call itself (``gemm_nt_fp8``, or ``gemm_nt_fp8_config`` when a configuration is given); returns
    its code without raising."""
    lib = load_library()
    if config is None:
        return int(lib.gemm_nt_fp8(_ptr(a), _ptr(b), _ptr(c), int(M), int(N), int(K), _stream_handle(stream), int(out_dtype)))
    return int(lib.gemm_nt_fp8_config(_ptr(a), _ptr(b), _ptr(c), int(M), int(N), int(K), _stream_handle(stream), int(out_dtype), int(config)))


def gemm_nt_fp8(a, b, c, M, N, K, stream=None, out_dtype=FP16, config=None) -> None:
    """``gemm_nt_fp8(a, b, c, M, N, K, stream, out_dtype)`` of the C ABI: ``C = A B^T`` for E4M3 bytes
    ``a`` [M,K], ``b`` [N,K] and a 16-bit ``c`` [M,N] of type ``out_dtype``.  Asynchronous.  With ``config``
    the call goes to ``gemm_nt_fp8_config``."""
    rc = gemm_nt_fp8_raw(a, b, c, M, N, K, stream, out_dtype, config)
    if rc != 0:
        raise GemmNtError(rc, load_library().gemm_nt_strerror(rc).decode())


def gemm_fp8_tile_params() -> dict:
    lib = load_library()
    return {"BM": lib.gemm_nt_fp8_tile_param(0), "BN": lib.gemm_nt_fp8_tile_param(1), "BK": lib.gemm_nt_fp8_tile_param(2),
            "stages": lib.gemm_nt_fp8_tile_param(3), "threads": lib.gemm_nt_fp8_tile_param(4)}

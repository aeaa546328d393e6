"""The C-ABI library loads on a machine without a GPU, exports every symbol the header
declares, and rejects bad arguments before touching HIP."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "attn_fwd.h")
GEMM_HEADER = os.path.join(ROOT, "include", "gemm_nt.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2510_14719_amd import binding
    return binding.load_library()


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(attn_fwd\w*)\s*\(", src)))


def test_header_symbols_are_exported(lib):
    names = declared_functions()
    assert {"attn_fwd", "attn_fwd_f16", "attn_fwd_bf16", "attn_fwd_strerror", "attn_fwd_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), "library does not export %s" % n


def test_version_and_strerror(lib):
    assert lib.attn_fwd_version() >= 100
    for code in range(-8, 1):
        text = lib.attn_fwd_strerror(code)
        assert text and len(text) > 3
    assert lib.attn_fwd_strerror(0) == b"success"


def test_tile_params(lib):
    for d in (64, 128):
        bm, bn, st, th = (lib.attn_fwd_tile_param(d, 0, w) for w in range(4))
        assert bm % 32 == 0 and bn % 32 == 0 and st >= 3 and th % 64 == 0
        assert st * 2 * bn * d * 2 <= 160 * 1024   # the LDS ring fits one CU
    assert lib.attn_fwd_tile_param(96, 0, 0) == -1
    assert lib.attn_fwd_tile_param(128, 0, 9) == -1


def test_argument_validation_needs_no_gpu(lib):
    # fake, aligned, non-overlapping addresses: validation never dereferences them
    q, k, v, o, l = 0x10000000, 0x20000000, 0x30000000, 0x40000000, 0x50000000
    f = lib.attn_fwd_check_args
    ok = (q, k, v, o, l, 2, 4, 1024, 128, 0.088, 0)
    assert f(*ok) == 0
    assert f(0, k, v, o, l, 2, 4, 1024, 128, 0.088, 0) == -1
    assert f(q, k, v, o, 0, 2, 4, 1024, 128, 0.088, 0) == -1
    assert f(q, k, v, o, l, 0, 4, 1024, 128, 0.088, 0) == -2
    assert f(q, k, v, o, l, 2, 4, 0, 128, 0.088, 0) == -2
    assert f(q, k, v, o, l, 2, 4, 1024, 96, 0.088, 0) == -2
    assert f(q, k, v, o, l, 2, 4, 1024, 128, 0.088, 2) == -2
    for bad in (0.0, -1.0, float("nan"), float("inf")):
        assert f(q, k, v, o, l, 2, 4, 1024, 128, bad, 0) == -3
    assert f(q + 8, k, v, o, l, 2, 4, 1024, 128, 0.088, 0) == -4
    assert f(q, k, v, o, l + 4, 2, 4, 1024, 128, 0.088, 0) == -4
    assert f(q, k, v, o, l, 1, 1, 2 ** 23, 128, 0.088, 0) == -5
    assert f(q, k, v, q, l, 2, 4, 1024, 128, 0.088, 0) == -7
    assert f(q, k, v, k + 16, l, 2, 4, 1024, 128, 0.088, 0) == -7


def test_fp8_argument_validation_needs_no_gpu(lib):
    q, k, v, o, l = 0x10000000, 0x20000000, 0x30000000, 0x40000000, 0x50000000
    f = lib.attn_fwd_fp8_check_args
    assert f(q, k, v, o, l, 2, 4, 1024, 128, 0.088, 0) == 0
    assert f(q, k, v, o, l, 2, 4, 1024, 64, 0.088, 1) == 0
    assert f(q, 0, v, o, l, 2, 4, 1024, 128, 0.088, 0) == -1
    assert f(q, k, v, o, l, 2, 0, 1024, 128, 0.088, 0) == -2
    assert f(q, k, v, o, l, 2, 4, 1024, 256, 0.088, 0) == -2
    assert f(q, k, v, o, l, 2, 4, 1024, 128, 0.088, 2) == -2       # O is fp16 or bf16
    assert f(q, k, v, o, l, 2, 4, 1024, 128, -0.5, 0) == -3
    assert f(q, k + 4, v, o, l, 2, 4, 1024, 128, 0.088, 0) == -4
    assert f(q, k, v, o, l, 1, 1, 2 ** 23, 128, 0.088, 0) == -5
    # O has two bytes per element, the inputs one: 2*4*1024*128 = 1 MiB of input, 2 MiB of output
    assert f(q, k, v, q, l, 2, 4, 1024, 128, 0.088, 0) == -7
    assert f(q, k, v, q - (2 << 20) + 16, l, 2, 4, 1024, 128, 0.088, 0) == -7
    assert f(q, k, v, q - (2 << 20), l, 2, 4, 1024, 128, 0.088, 0) == 0
    assert f(q, k, v, q + (1 << 20), l, 2, 4, 1024, 128, 0.088, 0) == 0
    assert lib.attn_fwd_fp8(None, None, None, None, None, 1, 1, 64, 128, 0.125, 0, None, 0) == -1
    for d in (64, 128):
        bm, bn, st, th = (lib.attn_fwd_fp8_tile_param(d, w) for w in range(4))
        assert bm == 256 and bn % 64 == 0 and th == 512
        assert st * 2 * bn * d <= 160 * 1024
    assert lib.attn_fwd_fp8_tile_param(96, 0) == -1


def test_entry_points_return_argument_errors_without_launching(lib):
    # the full entry points run the same validation first; with a NULL pointer no HIP call is made
    assert lib.attn_fwd_f16(None, None, None, None, None, 1, 1, 64, 64, 0.125, 0, None) == -1
    assert lib.attn_fwd_bf16(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 1, 1, 64, 48, 0.125, 0, None) == -2
    assert lib.attn_fwd(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 1, 1, 64, 64, 0.125, 0, None, 7) == -2


def test_mfma_probe_validation_needs_no_gpu(lib):
    f = lib.attn_fwd_mfma_probe
    assert f(None, 256, 100, 1, 0, None) == -1
    assert f(0x10000000, 0, 100, 1, 0, None) == -2
    assert f(0x10000000, 70000, 100, 1, 0, None) == -2
    assert f(0x10000000, 256, 0, 1, 0, None) == -2
    assert f(0x10000000, 256, 100, 1, 5, None) == -2
    assert f(0x10000002, 256, 100, 1, 0, None) == -4
    assert lib.attn_fwd_mfma_probe_sink_floats(256) == 256 * 512
    assert lib.attn_fwd_mfma_probe_sink_floats(0) == -1
    # 8 waves x iters x 8 MFMAs x 2*32*32*16 flops per workgroup
    assert lib.attn_fwd_mfma_probe_flops(2, 10) == 2 * 8 * 10 * 8 * 32768.0
    assert lib.attn_fwd_mfma_probe_flops(0, 10) == 0.0
    lib.attn_fwd_mfma_probe_flops_of.restype = ctypes.c_double
    assert lib.attn_fwd_mfma_probe_flops_of(2, 10, 1) == 2 * 8 * 10 * 8 * 32768.0
    assert lib.attn_fwd_mfma_probe_flops_of(2, 10, 2) == 2 * 8 * 10 * 8 * 4 * 32768.0     # 32x32x64 on E4M3
    assert lib.attn_fwd_mfma_probe_flops_of(2, 10, 3) == 0.0
    assert f(0x10000002, 256, 100, 1, 2, None) == -4                                       # dtype 2 passes the dtype check


def test_gemm_header_symbols_are_exported(lib):
    src = re.sub(r"/\*.*?\*/", "", open(GEMM_HEADER).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(gemm_nt\w*)\s*\(", src)))
    assert {"gemm_nt", "gemm_nt_config", "gemm_nt_f16", "gemm_nt_bf16", "gemm_nt_check_args", "gemm_nt_strerror", "gemm_nt_tile_param",
            "gemm_nt_fp8", "gemm_nt_fp8_config", "gemm_nt_fp8_check_args", "gemm_nt_fp8_tile_param"} <= set(names)
    for n in names:
        assert hasattr(lib, n), "library does not export %s" % n


def test_gemm_argument_validation_needs_no_gpu(lib):
    a, b, c = 0x10000000, 0x20000000, 0x30000000
    f = lib.gemm_nt_check_args
    assert f(a, b, c, 256, 256, 64, 0) == 0
    assert f(a, b, c, 1, 1, 32, 1) == 0
    assert f(0, b, c, 256, 256, 64, 0) == -1
    assert f(a, b, 0, 256, 256, 64, 0) == -1
    assert f(a, b, c, 0, 256, 64, 0) == -2
    assert f(a, b, c, 256, 0, 64, 0) == -2
    assert f(a, b, c, 256, 256, 0, 0) == -2
    assert f(a, b, c, 256, 256, 48, 0) == -2          # K must be a multiple of 32
    assert f(a, b, c, 256, 256, 64, 2) == -2
    assert f(a + 8, b, c, 256, 256, 64, 0) == -4
    assert f(a, b, c + 1, 256, 256, 64, 0) == -4
    assert f(a, b, c, 65536, 256, 16384, 0) == -5     # 2 GiB of A
    assert f(a, b, a, 256, 256, 64, 0) == -7
    assert f(a, b, b + 64, 256, 256, 64, 0) == -7
    # the entry points run the same validation first
    assert lib.gemm_nt(None, None, None, 1, 1, 32, None, 0) == -1
    assert lib.gemm_nt_f16(a, b, c, 8, 8, 31, None) == -2
    assert lib.gemm_nt_bf16(a, b, c, 8, 8, 64 + 8, None) == -2
    assert lib.gemm_nt_config(a, b, c, 8, 8, 64, None, 0, 5) == -2        # unknown configuration
    assert lib.gemm_nt_config(a, b, None, 8, 8, 64, None, 0, 2) == -1
    for code in range(-8, 1):
        assert len(lib.gemm_nt_strerror(code)) > 3
    bm, bn, bk, st, th = (lib.gemm_nt_tile_param(w) for w in range(5))
    assert st * (bm + bn) * bk * 2 <= 160 * 1024 and th % 64 == 0 and lib.gemm_nt_tile_param(9) == -1


def test_gemm_fp8_argument_validation_needs_no_gpu(lib):
    a, b, c = 0x10000000, 0x20000000, 0x30000000
    f = lib.gemm_nt_fp8_check_args
    assert f(a, b, c, 256, 256, 64, 0) == 0
    assert f(a, b, c, 1, 1, 128, 1) == 0
    assert f(0, b, c, 256, 256, 64, 0) == -1
    assert f(a, 0, c, 256, 256, 64, 0) == -1
    assert f(a, b, c, 0, 256, 64, 0) == -2
    assert f(a, b, c, 256, 256, 32, 0) == -2          # K must be a multiple of 64
    assert f(a, b, c, 256, 256, 96, 0) == -2
    assert f(a, b, c, 256, 256, 64, 2) == -2          # the result is fp16 or bf16
    assert f(a + 8, b, c, 256, 256, 64, 0) == -4
    assert f(a, b, c + 1, 256, 256, 64, 0) == -4
    assert f(a, b, c, 131072, 256, 16384, 0) == -5    # 2 GiB of A
    assert f(a, 0x100000000, 0x200000000, 65536, 256, 16384, 0) == 0      # 1 GiB of bytes is fine
    assert f(a, b, a, 256, 256, 64, 0) == -7
    assert f(a, b, b + 64, 256, 256, 64, 0) == -7
    assert lib.gemm_nt_fp8(None, None, None, 1, 1, 64, None, 0) == -1
    assert lib.gemm_nt_fp8(a, b, c, 8, 8, 63, None, 0) == -2
    assert lib.gemm_nt_fp8_config(a, b, c, 8, 8, 64, None, 0, 5) == -2     # unknown configuration
    assert lib.gemm_nt_fp8_config(a, b, c, 8, 8, 64, None, 0, -1) == -2
    assert lib.gemm_nt_fp8_config(None, b, c, 8, 8, 64, None, 0, 1) == -1
    bm, bn, bk, st, th = (lib.gemm_nt_fp8_tile_param(w) for w in range(5))
    assert st * (bm + bn) * bk <= 160 * 1024 and th % 64 == 0 and lib.gemm_nt_fp8_tile_param(9) == -1

"""Every schedule variant the sweep harness builds must compute the same thing: two non-default points per
operation (``sweep.TEST_VARIANTS``, built by ``__graft_entry__.build()`` /
``python -m paper_2510_14719_amd.sweep build --test-variants``) are loaded through the C ABI and compared with the
CPU oracle, within the library's tolerances: whole small shapes element by element, and sampled rows or entries
of a workload that is large enough for the steady state of every loop."""
import ctypes
import math
import os

import numpy as np
import pytest

from paper_2510_14719_amd import inputs as I, sweep

pytestmark = pytest.mark.gpu

TOL_O_MAX, TOL_O_MEAN, TOL_LSE = 2e-2, 2e-3, 1e-2      # the benchmark spec's tolerances for N(0,1) inputs


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "the gpu tests need a GPU"
    from paper_2510_14719_amd import binding
    from oracle import attn_ref, gemm_ref
    binding.load_library()          # torch's HIP runtime first, as for the product library
    attn_ref.build()
    gemm_ref.build()
    return torch, attn_ref, gemm_ref


def _lib(op, point):
    path = sweep.variant_path(op, point)
    assert os.path.exists(path), "%s is missing: build it with `python -m paper_2510_14719_amd.sweep build --test-variants`" % path
    return sweep._load(path)


def _cases(op):
    return [pytest.param(op, p, id=sweep.variant_name(op, p)) for p in sweep.TEST_VARIANTS[op]]


def _attn(torch, lib, q, k, v, dtype, scale, causal, fp8=False):
    B, H, N, d = q.shape
    dq, dk, dv = (torch.from_numpy(x if fp8 else x.view(np.int16)).cuda() for x in (q, k, v))
    o = torch.full((B, H, N, d), 0x7FFF, dtype=torch.int16, device="cuda")
    lse = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    fn = lib.attn_fwd_fp8 if fp8 else lib.attn_fwd
    rc = fn(dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), o.data_ptr(), lse.data_ptr(), B, H, N, d, scale, int(causal), stream,
            0 if fp8 else dtype)
    torch.cuda.synchronize()
    assert rc == 0
    of = o.view(torch.bfloat16 if (dtype == I.BF16 and not fp8) else torch.float16).double().cpu().numpy()
    lf = lse.double().cpu().numpy()
    assert np.isfinite(of).all() and np.isfinite(lf).all(), "an element of O or LSE was never written"
    return of, lf


def _check(of, lf, o_ref, l_ref, what, tol=(TOL_O_MAX, TOL_O_MEAN, TOL_LSE)):
    eo, el = np.abs(of - o_ref), np.abs(lf - l_ref)
    msg = "%s: O max %.3e mean %.3e, LSE max %.3e" % (what, eo.max(), eo.mean(), el.max())
    print(msg, flush=True)
    assert eo.max() <= tol[0] and eo.mean() <= tol[1] and el.max() <= tol[2], msg


@pytest.mark.parametrize("op,point", _cases("attn_schedule") + _cases("attn_waves") + _cases("attn") + _cases("attn_causal"))
def test_attention_variants_against_the_oracle(env, op, point):
    torch, oracle, _ = env
    lib = _lib(op, point)
    print("variant %s" % sweep.variant_name(op, point), flush=True)
    # whole small shapes: several query tiles, ragged ends, both masks, both types (d = 128: the kernels the knobs touch)
    for (B, H, N, dtype, causal, seed) in [(2, 3, 577, I.FP16, False, 301), (1, 2, 1000, I.BF16, True, 302), (1, 2, 64, I.FP16, True, 303)]:
        q, k, v = I.make_qkv(B, H, N, 128, dtype, seed)
        scale = 1.0 / math.sqrt(128)
        o_ref, l_ref = oracle.attn_ref(q, k, v, dtype, scale, causal)
        of, lf = _attn(torch, lib, q, k, v, dtype, scale, causal)
        _check(of, lf, o_ref, l_ref, "N%d dtype%d causal%d" % (N, dtype, causal))
    # a workload long enough for the steady state of every loop, on sampled rows
    for name in (["c5"] if op == "attn_causal" else ["c3", "c5"]):
        w = I.WORKLOADS[name]
        q, k, v = I.make_workload(w)
        rows = I.sample_rows(w.B, w.H, w.N, 48, seed=w.seed + 17, always=[(0, 0, 0), (w.B - 1, w.H - 1, w.N - 1)])
        o_ref, l_ref = oracle.attn_ref_rows(q, k, v, w.dtype, rows, w.scale, w.causal)
        of, lf = _attn(torch, lib, q, k, v, w.dtype, w.scale, w.causal)
        idx = np.asarray(rows)
        _check(of[idx[:, 0], idx[:, 1], idx[:, 2]], lf[idx[:, 0], idx[:, 1], idx[:, 2]], o_ref, l_ref, name)


@pytest.mark.parametrize("op,point", _cases("attn_fp8"))
def test_fp8_attention_variants_against_the_oracle(env, op, point):
    torch, oracle, _ = env
    lib = _lib(op, point)
    print("variant %s" % sweep.variant_name(op, point), flush=True)
    # On a N(0,1) workload of this size the 8-bit path stays inside the 16-bit tolerances (the rounding of the
    # probabilities to E4M3, up to 2^-4 relative, averages out over thousands of keys).  Rows with few keys
    # (the small causal shape) or with a few dominant keys (f5: 5 % of the K rows scaled by 8) keep that rounding:
    # they get the looser tolerances of the library's smoke test.
    q, k, v = I.make_qkv(1, 2, 333, 128, I.E4M3, 304)
    scale = 1.0 / math.sqrt(128)
    o_ref, l_ref = oracle.attn_ref(q, k, v, I.E4M3, scale, True)
    of, lf = _attn(torch, lib, q, k, v, I.E4M3, scale, True, fp8=True)
    _check(of, lf, o_ref, l_ref, "fp8 N333 causal", tol=(1.5e-1, 8e-3, 7e-2))
    for name, tol in (("f3", (TOL_O_MAX, TOL_O_MEAN, TOL_LSE)), ("f5", (1.5e-1, 8e-3, 7e-2))):
        w = I.FP8_WORKLOADS[name]
        q, k, v = I.make_workload(w)
        rows = I.sample_rows(w.B, w.H, w.N, 48, seed=w.seed + 17, always=[(0, 0, 0), (w.B - 1, w.H - 1, w.N - 1)])
        o_ref, l_ref = oracle.attn_ref_rows(q, k, v, w.dtype, rows, w.scale, w.causal)
        of, lf = _attn(torch, lib, q, k, v, w.dtype, w.scale, w.causal, fp8=True)
        idx = np.asarray(rows)
        _check(of[idx[:, 0], idx[:, 1], idx[:, 2]], lf[idx[:, 0], idx[:, 1], idx[:, 2]], o_ref, l_ref, name, tol=tol)


@pytest.mark.parametrize("op,point", _cases("gemm") + _cases("gemm_fp8"))
def test_gemm_variants_against_the_oracle(env, op, point):
    torch, _, G = env
    lib = _lib(op, point)
    fp8 = op == "gemm_fp8"
    dtype = I.E4M3 if fp8 else I.FP16
    print("variant %s" % sweep.variant_name(op, point), flush=True)
    stream = torch.cuda.current_stream().cuda_stream
    for (M, N, K, full) in [(300, 520, 192, True), (1000, 777, 512, True), (4096, 4096, 2048, False)]:
        a, b = I.make_ab(M, N, K, dtype, seed=305 + K)
        da, db = (torch.from_numpy(x if fp8 else x.view(np.int16)).cuda() for x in (a, b))
        c = torch.full((M, N), 0x7FFF, dtype=torch.int16, device="cuda")
        fn = lib.gemm_nt_fp8 if fp8 else lib.gemm_nt
        assert fn(da.data_ptr(), db.data_ptr(), c.data_ptr(), M, N, K, stream, 0) == 0
        torch.cuda.synchronize()
        cf = c.view(torch.float16)
        assert bool(torch.isfinite(cf).all()), "an element of C was never written"
        if full:
            got, ref = cf.double().cpu().numpy(), G.gemm_nt(a, b, dtype)
            mag = None
            if fp8:
                mag = np.abs(torch.from_numpy(a).view(torch.float8_e4m3fn).double().numpy()) @ np.abs(torch.from_numpy(b).view(torch.float8_e4m3fn).double().numpy()).T
        else:
            idx = I.sample_entries(M, N, 64, seed=306 + K, always=[(0, 0), (M - 1, N - 1)])
            ii = np.asarray(idx)
            got, ref = cf[ii[:, 0], ii[:, 1]].double().cpu().numpy(), G.gemm_nt_samples(a, b, dtype, idx)
            mag = None
            if fp8:
                af = np.abs(torch.from_numpy(np.ascontiguousarray(a[ii[:, 0]])).view(torch.float8_e4m3fn).double().numpy())
                bf = np.abs(torch.from_numpy(np.ascontiguousarray(b[ii[:, 1]])).view(torch.float8_e4m3fn).double().numpy())
                mag = (af * bf).sum(axis=1)
        # the tolerances of the product's own tests: half an ulp of the fp16 result plus the accumulation term
        tol = 1.01 * 2.0 ** -11 * np.abs(ref) + (2.0 ** -14 * mag if fp8 else 2e-6 * K)
        worst = float((np.abs(got - ref) / tol).max())
        print("%dx%dx%d: worst err/tol %.3f" % (M, N, K, worst), flush=True)
        assert worst <= 1.0

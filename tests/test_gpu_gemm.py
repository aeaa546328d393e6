"""Parity of the HIP matrix product (through the C ABI) with the fp64 CPU oracle.

Tolerance (derived from the arithmetic: exact 16-bit x 16-bit products, fp32 accumulation over K terms,
one final rounding to 16 bit): |C_gpu - C_ref| <= 1.01 * u * |C_ref| + 2e-6 * K, with u = 2^-11 for
fp16 and 2^-8 for bf16 (half an ulp of the output); the second term bounds the accumulated fp32
rounding for N(0,1) operands (K * 2^-24 * sum|a||b| / sqrt(K) in the typical case) with a wide margin.
"""
import numpy as np
import pytest

from paper_2510_14719_amd import inputs as I

pytestmark = pytest.mark.gpu

U = {I.FP16: 2.0 ** -11, I.BF16: 2.0 ** -8}


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "the gpu tests need a GPU"
    from paper_2510_14719_amd import binding
    from oracle import gemm_ref
    binding.load_library()
    gemm_ref.build()
    return torch, binding, gemm_ref


def run_gpu(env, a, b, dtype, pad=512, config=None, finite=True):
    torch, binding, _ = env
    M, K = a.shape
    N = b.shape[0]
    da = torch.from_numpy(a.view(np.int16)).cuda()
    db = torch.from_numpy(b.view(np.int16)).cuda()
    buf = torch.full((M * N + 2 * pad,), 0x7FFF, dtype=torch.int16, device="cuda")
    c = buf[pad:pad + M * N]
    binding.gemm_nt(da, db, c, M, N, K, dtype=dtype, config=config)
    torch.cuda.synchronize()
    assert bool((buf[:pad] == 0x7FFF).all()) and bool((buf[pad + M * N:] == 0x7FFF).all()), "guard words overwritten"
    # (the buffer started out as NaN patterns: a finite C proves that every element was written)
    assert bool(torch.isfinite(c.view(torch.bfloat16 if dtype == I.BF16 else torch.float16)).all()) or not finite, "an element of C was never written"
    cc = c.view(torch.bfloat16 if dtype == I.BF16 else torch.float16).reshape(M, N)
    return cc


def check(c_gpu, c_ref, dtype, K, what):
    err = np.abs(c_gpu - c_ref)
    tol = 1.01 * U[dtype] * np.abs(c_ref) + 2e-6 * K
    worst = float((err / tol).max())
    print("%s: max err %.3e, worst err/tol %.3f" % (what, err.max(), worst), flush=True)
    assert np.isfinite(c_gpu).all(), what + ": non-finite C"
    assert worst <= 1.0, what


@pytest.mark.parametrize("dtype", [I.FP16, I.BF16])
@pytest.mark.parametrize("M,N,K", [(1, 1, 32), (5, 3, 64), (256, 256, 32), (256, 256, 96), (257, 255, 128), (300, 200, 160),
                                     (64, 1000, 256), (1000, 777, 512), (513, 1031, 64), (768, 512, 1024)])
def test_full_compare(env, M, N, K, dtype):
    _, _, G = env
    a, b = I.make_ab(M, N, K, dtype, seed=100 + M + N + K)
    print("case gemm M%d N%d K%d dtype%d" % (M, N, K, dtype), flush=True)
    ref = G.gemm_nt(a, b, dtype)
    c = run_gpu(env, a, b, dtype).double().cpu().numpy()
    check(c, ref, dtype, K, "full M%d N%d K%d" % (M, N, K))


@pytest.mark.parametrize("config", [1, 2, 3, 4])
@pytest.mark.parametrize("M,N,K,dtype", [(1, 1, 32, I.FP16), (257, 255, 64, I.BF16), (300, 520, 160, I.FP16), (640, 513, 1056, I.FP16),
                                           (256, 256, 2048, I.BF16)])
def test_every_kernel_configuration_in_full(env, M, N, K, dtype, config):
    # gemm_nt picks the configuration by K; each of the four kernels must handle every shape: one and two
    # K tiles, odd and even tile counts, overhanging tiles
    _, _, G = env
    a, b = I.make_ab(M, N, K, dtype, seed=600 + M + N + K)
    print("case gemm config%d M%d N%d K%d dtype%d" % (config, M, N, K, dtype), flush=True)
    ref = G.gemm_nt(a, b, dtype)
    c = run_gpu(env, a, b, dtype, config=config).double().cpu().numpy()
    check(c, ref, dtype, K, "config %d M%d N%d K%d" % (config, M, N, K))
    # the configurations add the K tiles of an entry in the same order: bit-identical results
    c1 = run_gpu(env, a, b, dtype, config=1).double().cpu().numpy()
    assert np.array_equal(c, c1)


def test_odd_n_uses_scalar_stores(env):
    _, _, G = env
    M, N, K = 130, 37, 96                     # N % 4 != 0: rows of C are not 8-byte aligned
    a, b = I.make_ab(M, N, K, I.FP16, seed=7)
    c = run_gpu(env, a, b, I.FP16).double().cpu().numpy()
    check(c, G.gemm_nt(a, b, I.FP16), I.FP16, K, "odd N")


def test_exact_small_integers(env):
    # products and sums of small integers are exact in fp32 and in the 16-bit output: bit-exact result
    torch, _, G = env
    rng = np.random.Generator(np.random.Philox(5))
    M, N, K = 300, 280, 64
    a = I.to_bits(rng.integers(-3, 4, size=(M, K)).astype(np.float32), I.FP16)
    b = I.to_bits(rng.integers(-3, 4, size=(N, K)).astype(np.float32), I.FP16)
    c = run_gpu(env, a, b, I.FP16).double().cpu().numpy()
    assert np.array_equal(c, G.gemm_nt(a, b, I.FP16))


@pytest.mark.parametrize("K", [256, 8192, 16384])
def test_paper_sweep_sizes_sampled(env, K):
    # M = N = 8192 (the benchmark's launch configuration), sampled entries against the oracle
    torch, binding, G = env
    M = N = 8192
    a, b = I.make_ab(M, N, K, I.FP16, seed=900 + K)
    print("case gemm sweep K%d" % K, flush=True)
    c = run_gpu(env, a, b, I.FP16)
    idx = I.sample_entries(M, N, 96, seed=901 + K, always=[(0, 0), (M - 1, N - 1), (0, N - 1), (M - 1, 0), (255, 256), (4096, 4095)])
    ref = G.gemm_nt_samples(a, b, I.FP16, idx)
    ii = np.asarray(idx)
    got = c[ii[:, 0], ii[:, 1]].double().cpu().numpy()
    check(got, ref, I.FP16, K, "sweep K%d" % K)
    # a property that holds at any size: the sum over each row of C equals A times the column sums of B^T
    bs = torch.from_numpy(b.view(np.int16)).cuda().view(torch.float16).double().sum(dim=0)       # [K]
    af = torch.from_numpy(a.view(np.int16)).cuda().view(torch.float16).double()
    row_sums_ref = (af @ bs).cpu().numpy()
    row_sums = c.double().sum(dim=1).cpu().numpy()
    # each of the N entries of a row carries at most half an ulp of rounding, of random sign
    bound = 6.0 * np.sqrt(N) * U[I.FP16] * np.sqrt(K) * 4 + 1e-6 * K * N ** 0.5
    assert np.abs(row_sums - row_sums_ref).max() <= bound


def test_repeat_runs_are_bit_identical_and_errors(env):
    torch, binding, _ = env
    a, b = I.make_ab(512, 512, 256, I.BF16, seed=9)
    c0 = run_gpu(env, a, b, I.BF16).clone()
    for _ in range(3):
        assert torch.equal(run_gpu(env, a, b, I.BF16), c0)
    t = torch.zeros(64 * 64 + 16, dtype=torch.float16, device="cuda")
    c = torch.zeros(64 * 64, dtype=torch.float16, device="cuda")
    assert binding.gemm_nt_raw(t, t, c, 64, 64, 64, None, 0) == 0
    assert binding.gemm_nt_raw(t, t, c, 64, 64, 40, None, 0) == -2
    assert binding.gemm_nt_raw(t[1:], t, c, 64, 64, 64, None, 0) == -4
    assert binding.gemm_nt_raw(t, t, t, 64, 64, 64, None, 0) == -7
    torch.cuda.synchronize()

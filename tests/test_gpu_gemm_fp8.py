"""Parity of the HIP matrix product on 8-bit-float (E4M3) operands (through the C ABI) with the fp64 CPU oracle.

Tolerance.  The product of two E4M3 values (4 significant bits each) is exact in fp32, so the result
differs from the exact one only by the summation and by the final rounding to 16 bit:
    |C_gpu - C_ref| <= 1.01 * u * |C_ref| + 2^-14 * S,      S = sum_k |A[m][k] B[n][k]|,
u = 2^-11 for an fp16 result and 2^-8 for bf16 (half an ulp).  The second term covers the summation:
the matrix core adds the 64 products of one instruction and the running sum in a frame that is narrower
than fp32 (a single instruction on random operands is off by up to 2^-16 S, measured), and the errors
of the K/64 instructions of an entry add up like a random walk, so relative to S, which grows with K,
they shrink (2^-16 S at K = 64, 2^-20 S at K = 16384, measured maxima over 10^5 entries).  2^-14 S leaves
a factor 4 at the smallest K and is still far below a single wrong term: one misplaced 16-byte column
of a fragment changes an entry by about 4 typical products, i.e. by 2^-4 S at K = 64 and 2^-12 S at
K = 16384.  Integer-valued operands, whose sums are exact in any frame, must match bit for bit.
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


def run_gpu(env, a, b, out_dtype, pad=512, config=None, finite=True):
    torch, binding, _ = env
    M, K = a.shape
    N = b.shape[0]
    da, db = torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda()
    buf = torch.full((M * N + 2 * pad,), 0x7FFF, dtype=torch.int16, device="cuda")
    c = buf[pad:pad + M * N]
    binding.gemm_nt_fp8(da, db, c, M, N, K, out_dtype=out_dtype, config=config)
    torch.cuda.synchronize()
    assert bool((buf[:pad] == 0x7FFF).all()) and bool((buf[pad + M * N:] == 0x7FFF).all()), "guard words overwritten"
    # (the buffer started out as NaN patterns: a finite C proves that every element was written)
    assert bool(torch.isfinite(c.view(torch.bfloat16 if out_dtype == I.BF16 else torch.float16)).all()) or not finite, "an element of C was never written"
    return c.view(torch.bfloat16 if out_dtype == I.BF16 else torch.float16).reshape(M, N)


def magnitudes(env, x):
    """|x| of E4M3 patterns as float64, decoded by torch (not by the oracle)."""
    torch = env[0]
    return torch.from_numpy(np.ascontiguousarray(x)).view(torch.float8_e4m3fn).to(torch.float64).abs().numpy()


def check(c_gpu, c_ref, s_abs, out_dtype, what):
    err = np.abs(c_gpu - c_ref)
    tol = 1.01 * U[out_dtype] * np.abs(c_ref) + 2.0 ** -14 * s_abs + 1e-30
    worst = float((err / tol).max())
    print("%s: max err %.3e, worst err/tol %.3f" % (what, err.max(), worst), flush=True)
    assert np.isfinite(c_gpu).all(), what + ": non-finite C"
    assert worst <= 1.0, what


@pytest.mark.parametrize("out_dtype", [I.FP16, I.BF16])
@pytest.mark.parametrize("M,N,K", [(1, 1, 64), (5, 3, 128), (256, 256, 64), (256, 256, 192), (257, 255, 128), (300, 200, 320),
                                     (64, 1000, 256), (1000, 777, 512), (513, 1031, 64), (768, 512, 1024)])
def test_full_compare(env, M, N, K, out_dtype):
    _, _, G = env
    a, b = I.make_ab(M, N, K, I.E4M3, seed=300 + M + N + K)
    print("case gemm_fp8 M%d N%d K%d out%d" % (M, N, K, out_dtype), flush=True)
    ref = G.gemm_nt(a, b, I.E4M3)
    c = run_gpu(env, a, b, out_dtype).double().cpu().numpy()
    check(c, ref, magnitudes(env, a) @ magnitudes(env, b).T, out_dtype, "full M%d N%d K%d" % (M, N, K))


@pytest.mark.parametrize("config", [1, 2, 3, 4])
@pytest.mark.parametrize("M,N,K", [(1, 1, 64), (257, 255, 128), (300, 520, 320), (640, 513, 2112), (256, 256, 2048)])
def test_every_kernel_configuration_in_full(env, M, N, K, config):
    # gemm_nt_fp8 picks the configuration by K (1 below 2048, 4 from there on); each of the four kernels
    # must handle every shape: one and two K tiles, odd and even tile counts, overhanging tiles
    _, _, G = env
    a, b = I.make_ab(M, N, K, I.E4M3, seed=500 + M + N + K)
    print("case gemm_fp8 config%d M%d N%d K%d" % (config, M, N, K), flush=True)
    ref = G.gemm_nt(a, b, I.E4M3)
    c = run_gpu(env, a, b, I.FP16, config=config).double().cpu().numpy()
    check(c, ref, magnitudes(env, a) @ magnitudes(env, b).T, I.FP16, "config %d M%d N%d K%d" % (config, M, N, K))
    # the configurations add the K tiles of an entry in the same order: bit-identical results, with or without
    # a configuration in the call
    c1 = run_gpu(env, a, b, I.FP16, config=1).double().cpu().numpy()
    c0 = run_gpu(env, a, b, I.FP16).double().cpu().numpy()
    assert np.array_equal(c, c1) and np.array_equal(c, c0)


def test_odd_n_uses_scalar_stores(env):
    _, _, G = env
    M, N, K = 130, 37, 192                    # N % 4 != 0: rows of C are not 8-byte aligned
    a, b = I.make_ab(M, N, K, I.E4M3, seed=7)
    c = run_gpu(env, a, b, I.FP16).double().cpu().numpy()
    check(c, G.gemm_nt(a, b, I.E4M3), magnitudes(env, a) @ magnitudes(env, b).T, I.FP16, "odd N")


def test_exact_small_integers(env):
    # products and sums of small integers are exact in every summation frame and in the 16-bit output
    _, _, G = env
    rng = np.random.Generator(np.random.Philox(5))
    M, N, K = 300, 280, 128
    a = I.to_bits(rng.integers(-3, 4, size=(M, K)).astype(np.float32), I.E4M3)
    b = I.to_bits(rng.integers(-3, 4, size=(N, K)).astype(np.float32), I.E4M3)
    c = run_gpu(env, a, b, I.FP16).double().cpu().numpy()
    assert np.array_equal(c, G.gemm_nt(a, b, I.E4M3))


def test_every_k_position_and_every_row_is_used_once(env):
    # A = one-hot rows scaled by distinct powers of two, B = a permutation-like pattern: each entry of C
    # is one product, so a k position read twice, skipped, or taken from the wrong row shows up exactly.
    _, _, G = env
    M, N, K = 256, 256, 256
    af = np.zeros((M, K), dtype=np.float32)
    bf = np.zeros((N, K), dtype=np.float32)
    for m in range(M):
        af[m, (7 * m + 3) % K] = 2.0 ** (m % 5 - 2)
    for n in range(N):
        bf[n, :] = 1.0 + 0.125 * ((np.arange(K) + 3 * n) % 8)          # exactly representable, row and k dependent
    a, b = I.to_bits(af, I.E4M3), I.to_bits(bf, I.E4M3)
    c = run_gpu(env, a, b, I.FP16).double().cpu().numpy()
    assert np.array_equal(c, G.gemm_nt(a, b, I.E4M3))
    assert np.array_equal(c, af.astype(np.float64) @ bf.astype(np.float64).T)


def test_extreme_values_do_not_overflow_the_accumulator(env):
    # all operands at the largest magnitude (448): every product is 200704, the sum over K = 64 is about
    # 1.3e7 in fp32; fp16 cannot hold it (inf by rounding), bf16 can
    torch, _, G = env
    M, N, K = 40, 72, 64
    a = np.full((M, K), 0x7E, dtype=np.uint8)
    b = np.full((N, K), 0x7E, dtype=np.uint8)
    b[::2] = 0xFE                                                          # alternate rows negative
    ref = G.gemm_nt(a, b, I.E4M3)
    c = run_gpu(env, a, b, I.BF16).double().cpu().numpy()
    assert np.abs(c - ref).max() <= 2.0 ** -8 * np.abs(ref).max()
    c16 = run_gpu(env, a, b, I.FP16, finite=False).double().cpu().numpy()
    assert np.isinf(c16).all() and np.array_equal(np.sign(c16), np.sign(ref))


def test_subnormal_operands_and_signed_zeros(env):
    # every product of two E4M3 subnormals (multiples of 2^-9) is a multiple of 2^-18 below 2^-12: the sums
    # over K = 64 stay exact in any summation frame that keeps 13 bits below its largest term, and in fp16
    _, _, G = env
    rng = np.random.Generator(np.random.Philox(21))
    M, N, K = 70, 90, 64
    a = rng.integers(0, 8, size=(M, K)).astype(np.uint8) | (rng.integers(0, 2, size=(M, K)).astype(np.uint8) << 7)
    b = rng.integers(0, 8, size=(N, K)).astype(np.uint8) | (rng.integers(0, 2, size=(N, K)).astype(np.uint8) << 7)
    ref = G.gemm_nt(a, b, I.E4M3)
    c = run_gpu(env, a, b, I.FP16).double().cpu().numpy()
    assert np.abs(ref).max() > 0 and np.array_equal(c, ref)


def test_nan_operands_poison_their_row_and_column_only(env):
    _, _, G = env
    M, N, K = 260, 300, 128
    a, b = I.make_ab(M, N, K, I.E4M3, seed=33)
    a[17, 5] = 0x7F                      # NaN in row 17 of A
    b[258, 127] = 0xFF                   # NaN in row 258 of B = column 258 of C
    ref = G.gemm_nt(a, b, I.E4M3)
    c = run_gpu(env, a, b, I.FP16, finite=False).double().cpu().numpy()
    want_nan = np.zeros((M, N), dtype=bool)
    want_nan[17, :] = True
    want_nan[:, 258] = True
    assert np.array_equal(np.isnan(ref), want_nan) and np.array_equal(np.isnan(c), want_nan)
    ok = ~want_nan
    s_abs = magnitudes(env, np.where(a == 0x7F, 0, a).astype(np.uint8)) @ magnitudes(env, np.where(b == 0xFF, 0, b).astype(np.uint8)).T
    err = np.abs(c[ok] - ref[ok])
    assert (err <= 1.01 * U[I.FP16] * np.abs(ref[ok]) + 2.0 ** -14 * s_abs[ok]).all()


@pytest.mark.parametrize("K", [256, 8192, 16384])
def test_paper_sweep_sizes_sampled(env, K):
    # M = N = 8192 (the benchmark's launch configuration), sampled entries against the oracle
    torch, binding, G = env
    M = N = 8192
    a, b = I.make_ab(M, N, K, I.E4M3, seed=900 + K)
    print("case gemm_fp8 sweep K%d" % K, flush=True)
    c = run_gpu(env, a, b, I.FP16)
    idx = I.sample_entries(M, N, 96, seed=901 + K, always=[(0, 0), (M - 1, N - 1), (0, N - 1), (M - 1, 0), (255, 256), (4096, 4095)])
    ref = G.gemm_nt_samples(a, b, I.E4M3, idx)
    ii = np.asarray(idx)
    got = c[ii[:, 0], ii[:, 1]].double().cpu().numpy()
    s_abs = (magnitudes(env, a[ii[:, 0]]) * magnitudes(env, b[ii[:, 1]])).sum(axis=1)
    check(got, ref, s_abs, I.FP16, "sweep K%d" % K)
    # a property that holds at any size: the sum over each row of C equals A times the column sums of B^T
    bs = torch.from_numpy(b).cuda().view(torch.float8_e4m3fn).double().sum(dim=0)       # [K]
    af = torch.from_numpy(a).cuda().view(torch.float8_e4m3fn).double()
    row_sums_ref = (af @ bs).cpu().numpy()
    row_sums = c.double().sum(dim=1).cpu().numpy()
    # each of the N entries of a row carries at most half an ulp of rounding, of random sign, plus the summation error
    bound = 6.0 * np.sqrt(N) * U[I.FP16] * np.sqrt(K) * 4 + 1e-4 * np.sqrt(K) * N ** 0.5
    assert np.abs(row_sums - row_sums_ref).max() <= bound


def test_repeat_runs_are_bit_identical_and_errors(env):
    torch, binding, _ = env
    a, b = I.make_ab(512, 512, 256, I.E4M3, seed=9)
    c0 = run_gpu(env, a, b, I.BF16).clone()
    for _ in range(3):
        assert torch.equal(run_gpu(env, a, b, I.BF16), c0)
    t = torch.zeros(64 * 64 + 16, dtype=torch.uint8, device="cuda")
    c = torch.zeros(64 * 64, dtype=torch.float16, device="cuda")
    assert binding.gemm_nt_fp8_raw(t, t, c, 64, 64, 64, None, 0) == 0
    assert binding.gemm_nt_fp8_raw(t, t, c, 64, 64, 96, None, 0) == -2
    assert binding.gemm_nt_fp8_raw(t, t, c, 64, 64, 64, None, 2) == -2
    assert binding.gemm_nt_fp8_raw(t[1:], t, c, 64, 64, 64, None, 0) == -4
    assert binding.gemm_nt_fp8_raw(t, t, t, 64, 64, 64, None, 0) == -7
    torch.cuda.synchronize()

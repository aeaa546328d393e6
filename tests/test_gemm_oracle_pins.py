"""Pins of the NT matrix-product oracle against things other than itself: a hand-worked example,
exact rational arithmetic, closed forms, algebraic identities and a library routine fed by an
independent decoder.  A transposed operand, a dropped term or a wrong index fails at least one."""
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2510_14719_amd import inputs as I

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "gemm_nt_2x2.txt")


@pytest.fixture(scope="module")
def G():
    from oracle import gemm_ref
    gemm_ref.build()
    return gemm_ref


def bits_of(x, dtype):
    return I.to_bits(np.asarray(x, dtype=np.float32), dtype)


def read_golden():
    mats, cur = {}, None
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        parts = line.split()
        if parts[0] in "ABC" and len(parts) == 3 and parts[0].isalpha():
            cur = parts[0]
            mats[cur] = []
        else:
            mats[cur].append([float(x) for x in parts])
    return {k: np.array(v) for k, v in mats.items()}


@pytest.mark.parametrize("dtype", [I.FP16, I.BF16, I.E4M3])
def test_hand_worked_example(G, dtype):
    g = read_golden()
    c = G.gemm_nt(bits_of(g["A"], dtype), bits_of(g["B"], dtype), dtype)
    assert c.shape == (2, 3)
    assert np.array_equal(c, g["C"])


def test_decoders_on_known_patterns(G):
    f16 = np.array([0x0000, 0x8000, 0x3C00, 0xC000, 0x3555, 0x7BFF, 0x0001, 0x03FF, 0x0400], dtype=np.uint16)
    want = [0.0, -0.0, 1.0, -2.0, 0.333251953125, 65504.0, 2.0 ** -24, 1023 * 2.0 ** -24, 2.0 ** -14]
    got = G.decode(f16, I.FP16)
    assert np.array_equal(got, np.array(want)) and np.signbit(got[1])
    bf = np.array([0x3F80, 0xC000, 0x3DCD, 0x0080, 0x7F7F], dtype=np.uint16)
    want = [1.0, -2.0, 0.10009765625, 2.0 ** -126, (2 - 2.0 ** -7) * 2.0 ** 127]
    assert np.array_equal(G.decode(bf, I.BF16), np.array(want))
    # every finite fp16 pattern against numpy's own conversion
    allbits = np.arange(0x7C00, dtype=np.uint16)
    assert np.array_equal(G.decode(allbits, I.FP16), allbits.view(np.float16).astype(np.float64))


def test_e4m3_decoder_against_torch_and_the_format_table(G):
    import torch
    allbits = np.arange(256, dtype=np.uint8)
    got = G.decode(allbits, I.E4M3)
    want = torch.from_numpy(allbits).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    nan = np.isnan(want)
    assert nan.sum() == 2 and np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan]) and np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))
    table = os.path.join(os.path.dirname(GOLDEN), "e4m3_values.txt")
    for line in open(table):
        if line.strip() and not line.startswith("#"):
            pat, val = line.split()
            g = G.decode(np.array([int(pat, 16)], dtype=np.uint8), I.E4M3)[0]
            assert (np.isnan(g) and val == "nan") or g == float(val)


@pytest.mark.parametrize("dtype", [I.FP16, I.BF16, I.E4M3])
def test_exact_rational_arithmetic_on_tiny_inputs(G, dtype):
    M, N, K = 3, 5, 7                       # all different: a transposed operand cannot go unnoticed
    a, b = I.make_ab(M, N, K, dtype, seed=11)
    c = G.gemm_nt(a, b, dtype)
    da, db = G.decode(a, dtype), G.decode(b, dtype)
    for m in range(M):
        for n in range(N):
            exact = sum(Fraction(float(da[m, k])) * Fraction(float(db[n, k])) for k in range(K))
            assert abs(Fraction(float(c[m, n])) - exact) <= abs(exact) * Fraction(1, 10 ** 13) + Fraction(1, 10 ** 15)


def test_identity_and_ones(G):
    K = 37
    a, _ = I.make_ab(11, 1, K, I.FP16, seed=12)
    eye = bits_of(np.eye(K), I.FP16)                      # B = I (N = K): C = A
    assert np.array_equal(G.gemm_nt(a, eye, I.FP16), G.decode(a, I.FP16))
    ones_a, ones_b = bits_of(np.ones((4, K)), I.BF16), bits_of(np.ones((9, K)), I.BF16)
    assert np.array_equal(G.gemm_nt(ones_a, ones_b, I.BF16), np.full((4, 9), float(K)))
    # a single 1 in B picks one column of A: C[m][n] = A[m][k0] for the row n whose 1 sits at k0
    sel = np.zeros((3, K)); sel[0, 5] = 1; sel[1, 0] = 1; sel[2, K - 1] = 1
    c = G.gemm_nt(a, bits_of(sel, I.FP16), I.FP16)
    da = G.decode(a, I.FP16)
    assert np.array_equal(c, da[:, [5, 0, K - 1]])


def test_rank_one(G):
    u = bits_of(np.arange(1, 7).reshape(6, 1) * 0.5, I.FP16)
    v = bits_of(np.arange(-4, 5).reshape(9, 1) * 0.25, I.FP16)
    want = (np.arange(1, 7).reshape(6, 1) * 0.5) @ (np.arange(-4, 5).reshape(1, 9) * 0.25)
    assert np.array_equal(G.gemm_nt(u, v, I.FP16), want)


@pytest.mark.parametrize("dtype", [I.FP16, I.BF16, I.E4M3])
def test_transpose_split_k_and_scaling_identities(G, dtype):
    M, N, K = 13, 21, 96
    a, b = I.make_ab(M, N, K, dtype, seed=13)
    c = G.gemm_nt(a, b, dtype)
    assert np.allclose(G.gemm_nt(b, a, dtype), c.T, rtol=1e-13, atol=1e-13)            # (A B^T)^T = B A^T
    k1 = 40
    parts = G.gemm_nt(a[:, :k1], b[:, :k1], dtype) + G.gemm_nt(a[:, k1:], b[:, k1:], dtype)
    assert np.allclose(parts, c, rtol=1e-13, atol=1e-12)                                # the sum over k splits
    a2 = bits_of(G.decode(a, dtype) * 2.0, dtype)                                        # exact in 16 bit
    assert np.array_equal(G.gemm_nt(a2, b, dtype), 2.0 * c)
    # rows of C depend on the matching rows of A only, columns on the matching rows of B only
    assert np.array_equal(G.gemm_nt(a[3:5], b, dtype), c[3:5])
    assert np.array_equal(G.gemm_nt(a, b[7:10], dtype), c[:, 7:10])


@pytest.mark.parametrize("dtype", [I.FP16, I.BF16, I.E4M3])
def test_against_library_matmul_with_independent_decoder(G, dtype):
    M, N, K = 70, 45, 300
    a, b = I.make_ab(M, N, K, dtype, seed=14)
    if dtype == I.FP16:
        da, db = a.view(np.float16).astype(np.float64), b.view(np.float16).astype(np.float64)
    elif dtype == I.E4M3:
        import torch
        da, db = (torch.from_numpy(x).view(torch.float8_e4m3fn).to(torch.float64).numpy() for x in (a, b))
    else:
        da = (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        db = (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    want = da @ db.T
    assert np.allclose(G.gemm_nt(a, b, dtype), want, rtol=1e-13, atol=1e-12)


def test_samples_match_full(G):
    M, N, K = 33, 29, 64
    a, b = I.make_ab(M, N, K, I.BF16, seed=15)
    c = G.gemm_nt(a, b, I.BF16)
    idx = I.sample_entries(M, N, 40, seed=16, always=[(0, 0), (M - 1, N - 1), (0, N - 1)])
    s = G.gemm_nt_samples(a, b, I.BF16, idx)
    assert np.array_equal(s, np.array([c[m, n] for m, n in idx]))
    with pytest.raises(RuntimeError):
        G.gemm_nt_samples(a, b, I.BF16, [(M, 0)])


def test_inputs_are_seeded_and_shaped():
    a, b = I.make_ab(8, 5, 16, I.FP16, seed=3)
    a2, b2 = I.make_ab(8, 5, 16, I.FP16, seed=3)
    assert a.shape == (8, 16) and b.shape == (5, 16) and a.dtype == np.uint16
    assert np.array_equal(a, a2) and np.array_equal(b, b2) and not np.array_equal(a[:5], b)
    assert I.sample_entries(8, 5, 6, seed=1) == I.sample_entries(8, 5, 6, seed=1)

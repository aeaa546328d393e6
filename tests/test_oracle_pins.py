"""Pins for the CPU oracle: every check here is fixed by the definition of
attention or by mathematics, not by the oracle's own code.

A dropped scale, a wrong sign, a transposed operand, an off-by-one causal mask,
a wrong log base or a wrong decoder each break at least one of these.
"""
import math
import os
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest
import scipy.special

from paper_2510_14719_amd import inputs as I

FP16, BF16 = I.FP16, I.BF16
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def np_decode(bits, dtype):
    """Library decode (numpy), independent of the oracle's own decoder."""
    bits = np.asarray(bits, dtype=np.uint16)
    if dtype == FP16:
        return bits.view(np.float16).astype(np.float64)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def bits_of(x, dtype):
    return I.to_bits(np.asarray(x, dtype=np.float32), dtype)


# ---------------------------------------------------------------- decoders
@pytest.mark.parametrize("dtype", [FP16, BF16])
def test_decoder_all_patterns(oracle, dtype):
    allbits = np.arange(65536, dtype=np.uint16)
    got = oracle.decode(allbits, dtype)
    want = np_decode(allbits, dtype)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


# ---------------------------------------------------------------- invariants of the definition
@pytest.mark.parametrize("dtype", [FP16, BF16])
@pytest.mark.parametrize("causal", [False, True])
def test_softmax_rows_sum_to_one(oracle, dtype, causal):
    q, k, v = I.make_qkv(2, 3, 37, 16, dtype, seed=11)
    _, _, p = oracle.attn_ref(q, k, v, dtype, 0.25, causal, return_p=True)
    assert np.all(p >= 0)
    assert np.max(np.abs(p.sum(-1) - 1.0)) < 1e-12
    if causal:
        iu = np.triu_indices(37, k=1)
        assert np.all(p[..., iu[0], iu[1]] == 0.0)


@pytest.mark.parametrize("causal", [False, True])
def test_constant_v_rows_return_that_row(oracle, causal):
    B, H, N, d = 1, 2, 33, 8
    q, k, _ = I.make_qkv(B, H, N, d, FP16, seed=12)
    row = np.linspace(-2, 2, d).astype(np.float32)
    v = bits_of(np.broadcast_to(row, (B, H, N, d)), FP16)
    o, _ = oracle.attn_ref(q, k, v, FP16, 0.7, causal)
    want = np_decode(bits_of(row, FP16), FP16)
    assert np.max(np.abs(o - want)) < 1e-12


@pytest.mark.parametrize("dtype", [FP16, BF16])
@pytest.mark.parametrize("causal", [False, True])
def test_zero_q_gives_mean_of_visible_v(oracle, dtype, causal):
    B, H, N, d = 2, 2, 29, 8
    _, k, v = I.make_qkv(B, H, N, d, dtype, seed=13)
    q = np.zeros((B, H, N, d), dtype=np.uint16)
    o, lse = oracle.attn_ref(q, k, v, dtype, 0.3, causal)
    vf = np_decode(v, dtype)
    for i in range(N):
        vis = i + 1 if causal else N
        assert np.max(np.abs(o[:, :, i] - vf[:, :, :vis].mean(axis=2))) < 1e-12
        assert np.max(np.abs(lse[:, :, i] - math.log(vis))) < 1e-12


def test_causal_row0_returns_v0_and_s00(oracle):
    B, H, N, d = 2, 2, 17, 8
    q, k, v = I.make_qkv(B, H, N, d, FP16, seed=14)
    scale = 0.37
    o, lse = oracle.attn_ref(q, k, v, FP16, scale, True)
    qf, kf, vf = (np_decode(x, FP16) for x in (q, k, v))
    assert np.array_equal(o[:, :, 0], vf[:, :, 0])
    for b in range(B):
        for h in range(H):
            s00 = scale * math.fsum(qf[b, h, 0] * kf[b, h, 0])
            assert abs(lse[b, h, 0] - s00) < 1e-12


def test_permuting_k_and_v_together_changes_nothing(oracle):
    B, H, N, d = 1, 2, 41, 8
    q, k, v = I.make_qkv(B, H, N, d, BF16, seed=15)
    perm = np.random.Generator(np.random.Philox(99)).permutation(N)
    o1, l1 = oracle.attn_ref(q, k, v, BF16, 0.5, False)
    o2, l2 = oracle.attn_ref(q, k[:, :, perm], v[:, :, perm], BF16, 0.5, False)
    assert np.max(np.abs(o1 - o2)) < 1e-12
    assert np.max(np.abs(l1 - l2)) < 1e-12
    # ... and permuting V alone does change it (the check above is not vacuous)
    o3, _ = oracle.attn_ref(q, k, v[:, :, perm], BF16, 0.5, False)
    assert np.max(np.abs(o1 - o3)) > 1e-3


def test_equal_k_rows_give_uniform_weights(oracle):
    B, H, N, d = 1, 1, 23, 8
    q, _, v = I.make_qkv(B, H, N, d, FP16, seed=16)
    krow = np.linspace(-1, 1, d).astype(np.float32)
    k = bits_of(np.broadcast_to(krow, (B, H, N, d)), FP16)
    o, lse = oracle.attn_ref(q, k, v, FP16, 0.9, False)
    vf, qf, kf = np_decode(v, FP16), np_decode(q, FP16), np_decode(k, FP16)
    assert np.max(np.abs(o - vf.mean(axis=2, keepdims=True))) < 1e-12
    s = 0.9 * (qf[0, 0] @ kf[0, 0, 0])
    assert np.max(np.abs(lse[0, 0] - (s + math.log(N)))) < 1e-12


def test_score_shift_moves_lse_only(oracle):
    """Append a feature: q gets 1, every k gets c/scale -> every score of a row grows by c."""
    B, H, N, d = 1, 2, 19, 8
    scale, c = 0.5, 3.0
    rng = np.random.Generator(np.random.Philox(17))
    qf = rng.standard_normal((B, H, N, d + 8), dtype=np.float32)
    kf = rng.standard_normal((B, H, N, d + 8), dtype=np.float32)
    vf = rng.standard_normal((B, H, N, d + 8), dtype=np.float32)
    qf[..., d:] = 0
    kf[..., d:] = 0
    q0, k0, v0 = bits_of(qf, FP16), bits_of(kf, FP16), bits_of(vf, FP16)
    qf[..., d] = 1.0
    kf[..., d] = c / scale
    q1, k1 = bits_of(qf, FP16), bits_of(kf, FP16)
    o0, l0 = oracle.attn_ref(q0, k0, v0, FP16, scale, False)
    o1, l1 = oracle.attn_ref(q1, k1, v0, FP16, scale, False)
    assert np.max(np.abs(o0 - o1)) < 1e-12
    assert np.max(np.abs(l1 - l0 - c)) < 1e-12


def test_one_hot_keys_select_value_rows(oracle):
    N = d = 16
    lam = 64.0
    perm = np.random.Generator(np.random.Philox(18)).permutation(N)
    kf = lam * np.eye(N, dtype=np.float32)
    qf = np.eye(N, dtype=np.float32)[perm]
    _, _, v = I.make_qkv(1, 1, N, d, FP16, seed=18)
    o, lse = oracle.attn_ref(bits_of(qf, FP16)[None, None], bits_of(kf, FP16)[None, None], v, FP16, 1.0, False)
    vf = np_decode(v, FP16)[0, 0]
    # weight of the wrong keys is (N-1) e^-64 relative to the right one
    assert np.max(np.abs(o[0, 0] - vf[perm])) < 1e-20 * 1e3 + 16 * math.exp(-lam) * 10
    assert np.max(np.abs(lse[0, 0] - lam)) < 1e-12


def test_split_keys_and_merge_with_lse(oracle):
    B, H, N, d = 1, 2, 48, 8
    q, k, v = I.make_qkv(B, H, N, d, BF16, seed=19)
    o, l = oracle.attn_ref(q, k, v, BF16, 0.4, False)
    h = 20

    def part(lo, hi):
        # all N queries against keys [lo, hi): pad the key set by calling row-wise on a
        # tensor whose N equals the key count would change the queries, so instead run
        # the square problem on a tensor made of the kept keys repeated for the queries.
        n = hi - lo
        os_, ls_ = [], []
        for i0 in range(0, N, n):
            qs = q[:, :, i0:i0 + n]
            pad = n - qs.shape[2]
            if pad:
                qs = np.concatenate([qs, np.zeros((B, H, pad, d), np.uint16)], axis=2)
            oo, ll = oracle.attn_ref(qs, k[:, :, lo:hi], v[:, :, lo:hi], BF16, 0.4, False)
            os_.append(oo)
            ls_.append(ll)
        return np.concatenate(os_, axis=2)[:, :, :N], np.concatenate(ls_, axis=2)[:, :, :N]

    o1, l1 = part(0, h)
    o2, l2 = part(h, N)
    lm = np.logaddexp(l1, l2)
    om = (np.exp(l1 - lm)[..., None] * o1 + np.exp(l2 - lm)[..., None] * o2)
    assert np.max(np.abs(lm - l)) < 1e-12
    assert np.max(np.abs(om - o)) < 1e-12


def test_two_key_logistic_golden(oracle):
    want = {}
    with open(os.path.join(GOLDEN, "two_key_logistic.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, val = line.split()
            want[name] = float(val)
    q = bits_of([[[[1.0], [1.0]]]], FP16)
    k = bits_of([[[[0.0], [1.0]]]], FP16)
    v = bits_of([[[[0.0], [1.0]]]], FP16)
    for dtype in (FP16, BF16):
        o, lse = oracle.attn_ref(q if dtype == FP16 else bits_of([[[[1.0], [1.0]]]], BF16),
                                 k if dtype == FP16 else bits_of([[[[0.0], [1.0]]]], BF16),
                                 v if dtype == FP16 else bits_of([[[[0.0], [1.0]]]], BF16),
                                 dtype, 1.0, False)
        assert np.max(np.abs(o - want["O"])) < 1e-15
        assert np.max(np.abs(lse - want["LSE"])) < 1e-15
    # the same two keys under a causal mask: row 0 sees only key 0
    o, lse = oracle.attn_ref(q, k, v, FP16, 1.0, True)
    assert o[0, 0, 0, 0] == 0.0 and lse[0, 0, 0] == 0.0
    assert abs(o[0, 0, 1, 0] - want["O"]) < 1e-15 and abs(lse[0, 0, 1] - want["LSE"]) < 1e-15


# ---------------------------------------------------------------- brute force, differently structured
def _brute_force(qf, kf, vf, scale, causal):
    """50-digit decimal arithmetic, exact rational dot products, no max subtraction:
    p_ij = 1 / sum_k exp(s_ik - s_ij),  LSE_i = ln sum_k exp(s_ik)."""
    getcontext().prec = 50
    N, d = qf.shape
    sc = Fraction(scale)
    O = np.zeros((N, d))
    L = np.zeros(N)
    for i in range(N):
        vis = range(i + 1) if causal else range(N)
        s = {}
        for j in vis:
            acc = Fraction(0)
            for t in range(d):
                acc += Fraction(float(qf[i, t])) * Fraction(float(kf[j, t]))
            acc *= sc
            s[j] = Decimal(acc.numerator) / Decimal(acc.denominator)
        tot = sum((s[j].exp() for j in vis), Decimal(0))
        L[i] = float(tot.ln())
        for t in range(d):
            acc = Decimal(0)
            for j in vis:
                pij = Decimal(1) / sum(((s[kk] - s[j]).exp() for kk in vis), Decimal(0))
                acc += pij * Decimal(float(vf[j, t]))
            O[i, t] = float(acc)
    return O, L


@pytest.mark.parametrize("dtype", [FP16, BF16])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("N,d", [(1, 4), (2, 1), (7, 3), (12, 5)])
def test_brute_force_tiny(oracle, dtype, causal, N, d):
    q, k, v = I.make_qkv(1, 2, N, d, dtype, seed=100 + N)
    scale = 0.4375  # exactly representable, so Fraction(scale) is what the oracle gets
    o, lse = oracle.attn_ref(q, k, v, dtype, scale, causal)
    qf, kf, vf = (np_decode(x, dtype) for x in (q, k, v))
    for h in range(2):
        O, L = _brute_force(qf[0, h], kf[0, h], vf[0, h], scale, causal)
        assert np.max(np.abs(o[0, h] - O)) < 1e-13
        assert np.max(np.abs(lse[0, h] - L)) < 1e-13


# ---------------------------------------------------------------- reduction to library routines
@pytest.mark.parametrize("dtype", [FP16, BF16])
@pytest.mark.parametrize("causal", [False, True])
def test_against_scipy_softmax_and_logsumexp(oracle, dtype, causal):
    B, H, N, d = 2, 3, 150, 64
    q, k, v = I.make_qkv(B, H, N, d, dtype, seed=21, peaky=True)
    scale = 1.0 / math.sqrt(d)
    o, lse = oracle.attn_ref(q, k, v, dtype, scale, causal)
    qf, kf, vf = (np_decode(x, dtype) for x in (q, k, v))
    s = scale * np.einsum("bhid,bhjd->bhij", qf, kf)
    if causal:
        s = np.where(np.tril(np.ones((N, N), dtype=bool)), s, -np.inf)
    want_o = np.einsum("bhij,bhjd->bhid", scipy.special.softmax(s, axis=-1), vf)
    want_l = scipy.special.logsumexp(s, axis=-1)
    assert np.max(np.abs(o - want_o)) < 1e-12
    assert np.max(np.abs(lse - want_l)) < 1e-12


# ---------------------------------------------------------------- the row-sampled entry point is the same definition
@pytest.mark.parametrize("causal", [False, True])
def test_rows_entry_point_matches_full(oracle, causal):
    B, H, N, d = 2, 2, 70, 16
    q, k, v = I.make_qkv(B, H, N, d, FP16, seed=22)
    o, lse = oracle.attn_ref(q, k, v, FP16, 0.25, causal)
    rows = I.sample_rows(B, H, N, 25, seed=5, always=[(0, 0, 0), (B - 1, H - 1, N - 1)])
    orows, lrows = oracle.attn_ref_rows(q, k, v, FP16, rows, 0.25, causal)
    for r, (b, h, i) in enumerate(rows):
        assert np.array_equal(orows[r], o[b, h, i])
        assert lrows[r] == lse[b, h, i]


def test_bad_arguments_are_rejected(oracle):
    q, k, v = I.make_qkv(1, 1, 4, 4, FP16, seed=23)
    with pytest.raises(RuntimeError):
        oracle.attn_ref_rows(q, k, v, FP16, [(0, 0, 4)], 1.0, False)
    with pytest.raises(TypeError):
        oracle.attn_ref(q.astype(np.float32), k, v, FP16, 1.0, False)

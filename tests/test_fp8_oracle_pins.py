"""Pins for the 8-bit-float (E4M3) side of the CPU oracle.

The arithmetic of the oracle is the same for every element type and is pinned in
``test_oracle_pins.py``; what E4M3 adds is a decoder, byte-wide storage and the
probability rows of the sampled entry point.  Everything here is fixed by the format
definition, by a library decoder or by mathematics.
"""
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

from paper_2510_14719_amd import inputs as I

E4M3 = I.E4M3
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def torch_decode(bits):
    """Library decode (torch's float8_e4m3fn), independent of the oracle's own decoder."""
    b = np.ascontiguousarray(bits, dtype=np.uint8)
    return torch.from_numpy(b).view(torch.float8_e4m3fn).to(torch.float64).numpy()


def test_decoder_against_the_format_table(oracle):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "e4m3_values.txt")) if l.strip() and not l.startswith("#")]
    bits = np.array([int(r[0], 16) for r in rows], dtype=np.uint8)
    got = oracle.decode(bits, E4M3)
    for (pat, val), g in zip(rows, got):
        want = float(val)
        if math.isnan(want):
            assert math.isnan(g), pat
        else:
            assert g == want and math.copysign(1.0, g) == math.copysign(1.0, want), pat


def test_decoder_all_patterns_against_torch(oracle):
    allbits = np.arange(256, dtype=np.uint8)
    got, want = oracle.decode(allbits, E4M3), torch_decode(allbits)
    nan = np.isnan(want)
    assert nan.sum() == 2
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_rounding_to_e4m3_matches_torch_and_saturates():
    rng = np.random.Generator(np.random.Philox(3))
    x = np.concatenate([rng.standard_normal(100000, dtype=np.float32) * np.float32(s) for s in (1.0, 0.01, 30.0, 0.002)])
    x[:12] = [0.0, -0.0, 1.0625, 1.1875, 17.0, 19.0, 2.0 ** -10, 1.5 * 2.0 ** -9, 2.5 * 2.0 ** -9, 448.0, 463.0, -2.5]
    want = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(I.f32_to_e4m3_bits(x), want)
    # ties go to the even code: 1.0625 -> 1.0, 1.1875 -> 1.25, 17 -> 16, 19 -> 20
    assert I.f32_to_e4m3_bits(np.float32([1.0625, 1.1875, 17.0, 19.0])).tolist() == [0x38, 0x3A, 0x58, 0x5A]
    # beyond the largest finite the generator saturates (never NaN)
    assert I.f32_to_e4m3_bits(np.float32([464.0, 1e9, -1e9])).tolist() == [0x7E, 0x7E, 0xFE]


def test_two_key_logistic_closed_form_in_e4m3(oracle):
    """The hand-worked case of ``golden/two_key_logistic.txt`` (q = [1, 1], k = [0, 1], v = [0, 1], d = 1,
    scale 1: O = logistic(1), LSE = softplus(1)); every input is exactly representable in E4M3."""
    vals = dict(l.split() for l in open(os.path.join(GOLDEN, "two_key_logistic.txt")) if l.strip() and not l.startswith("#"))
    one, zero = 0x38, 0x00
    q = np.array([one, one], dtype=np.uint8).reshape(1, 1, 2, 1)
    k = np.array([zero, one], dtype=np.uint8).reshape(1, 1, 2, 1)
    v = np.array([zero, one], dtype=np.uint8).reshape(1, 1, 2, 1)
    o, lse = oracle.attn_ref(q, k, v, E4M3, 1.0, False)
    assert np.max(np.abs(o - float(vals["O"]))) < 1e-15
    assert np.max(np.abs(lse - float(vals["LSE"]))) < 1e-15
    # causal: row 0 sees only key 0 (O = v_0 = 0, LSE = s_00 = 0), row 1 is the case above
    o, lse = oracle.attn_ref(q, k, v, E4M3, 1.0, True)
    assert o[0, 0, 0, 0] == 0.0 and lse[0, 0, 0] == 0.0
    assert abs(o[0, 0, 1, 0] - float(vals["O"])) < 1e-15 and abs(lse[0, 0, 1] - float(vals["LSE"])) < 1e-15


@pytest.mark.parametrize("causal", [False, True])
def test_zero_q_gives_mean_of_visible_v(oracle, causal):
    B, H, N, d = 2, 2, 29, 8
    _, k, v = I.make_qkv(B, H, N, d, E4M3, seed=31)
    q = np.zeros((B, H, N, d), dtype=np.uint8)
    o, lse = oracle.attn_ref(q, k, v, E4M3, 0.3, causal)
    vf = torch_decode(v)
    for i in range(N):
        vis = i + 1 if causal else N
        assert np.max(np.abs(o[:, :, i] - vf[:, :, :vis].mean(axis=2))) < 1e-12
        assert np.max(np.abs(lse[:, :, i] - math.log(vis))) < 1e-12


@pytest.mark.parametrize("causal", [False, True])
def test_against_scipy_softmax_and_logsumexp(oracle, causal):
    B, H, N, d = 2, 3, 150, 64
    q, k, v = I.make_qkv(B, H, N, d, E4M3, seed=32, peaky=True)
    scale = 1.0 / math.sqrt(d)
    o, lse = oracle.attn_ref(q, k, v, E4M3, scale, causal)
    qf, kf, vf = (torch_decode(x) for x in (q, k, v))
    s = scale * np.einsum("bhid,bhjd->bhij", qf, kf)
    if causal:
        s = np.where(np.tril(np.ones((N, N), dtype=bool)), s, -np.inf)
    want_o = np.einsum("bhij,bhjd->bhid", scipy.special.softmax(s, axis=-1), vf)
    want_l = scipy.special.logsumexp(s, axis=-1)
    assert np.max(np.abs(o - want_o)) < 1e-12
    assert np.max(np.abs(lse - want_l)) < 1e-12


def test_same_values_in_fp16_and_e4m3_give_the_same_result(oracle):
    """Every E4M3 value is an fp16 value: feeding the same numbers through either decoder changes nothing."""
    B, H, N, d = 1, 2, 40, 16
    q8, k8, v8 = I.make_qkv(B, H, N, d, E4M3, seed=33)
    q16, k16, v16 = (torch_decode(x).astype(np.float16).view(np.uint16) for x in (q8, k8, v8))
    o8, l8 = oracle.attn_ref(q8, k8, v8, E4M3, 0.25, True)
    o16, l16 = oracle.attn_ref(q16, k16, v16, I.FP16, 0.25, True)
    assert np.array_equal(o8, o16) and np.array_equal(l8, l16)


@pytest.mark.parametrize("causal", [False, True])
def test_rows_entry_point_and_its_probability_rows(oracle, causal):
    B, H, N, d = 2, 2, 70, 16
    q, k, v = I.make_qkv(B, H, N, d, E4M3, seed=34)
    o, lse, p = oracle.attn_ref(q, k, v, E4M3, 0.25, causal, return_p=True)
    rows = I.sample_rows(B, H, N, 25, seed=5, always=[(0, 0, 0), (B - 1, H - 1, N - 1)])
    orows, lrows, prows = oracle.attn_ref_rows(q, k, v, E4M3, rows, 0.25, causal, return_p=True)
    vf = torch_decode(v)
    for r, (b, h, i) in enumerate(rows):
        assert np.array_equal(orows[r], o[b, h, i])
        assert lrows[r] == lse[b, h, i]
        assert np.array_equal(prows[r], p[b, h, i])
        assert abs(prows[r].sum() - 1.0) < 1e-12
        assert np.max(np.abs(prows[r] @ vf[b, h] - orows[r])) < 1e-12     # O is the P-weighted mean of the V rows


def test_storage_type_is_checked(oracle):
    q, k, v = I.make_qkv(1, 1, 4, 4, E4M3, seed=35)
    with pytest.raises(TypeError):
        oracle.attn_ref(q.astype(np.uint16), k, v, E4M3, 1.0, False)
    q16, k16, v16 = I.make_qkv(1, 1, 4, 4, I.FP16, seed=35)
    with pytest.raises(TypeError):
        oracle.attn_ref(q16.view(np.uint8).reshape(1, 1, 4, 8), k16, v16, I.FP16, 1.0, False)

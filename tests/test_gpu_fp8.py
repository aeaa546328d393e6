"""Parity of the 8-bit-float attention kernel (through the C ABI) with the fp64 CPU oracle.

The oracle computes the exact definition on the decoded E4M3 inputs.  The kernel additionally
rounds the probabilities to E4M3 before the second contraction, an approximation whose worst case
is derived in ``gpu_util.fp8_bounds``; every output element must lie inside that bound, the mean
error well inside it, and on the large N(0,1) workloads (many keys per row, the errors average
out) the 16-bit tolerances hold as well.
"""
import math

import numpy as np
import pytest

from paper_2510_14719_amd import inputs as I

pytestmark = pytest.mark.gpu
E4M3 = I.E4M3


@pytest.fixture(scope="module")
def G():
    import torch
    assert torch.cuda.is_available(), "the gpu tests need a GPU"
    from tests import gpu_util
    from paper_2510_14719_amd import binding
    binding.load_library()   # fails loudly if the extension was not built
    return gpu_util


def _full(G, oracle, B, H, N, d, causal, seed, out_dtype=I.FP16, scale=None, peaky=False, what="", qkv=None):
    q, k, v = I.make_qkv(B, H, N, d, E4M3, seed, peaky=peaky) if qkv is None else qkv
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    print("case %s B%d H%d N%d d%d out%d causal%d seed%d" % (what, B, H, N, d, out_dtype, causal, seed), flush=True)
    o_ref, l_ref, p = oracle.attn_ref(q, k, v, E4M3, scale, causal, return_p=True)
    o, l = G.run_gpu_fp8(q, k, v, out_dtype, scale, causal)
    bo, bl = G.fp8_bounds(p, G.e4m3_to_f64(v), o_ref, out_dtype)
    G.check_fp8(o, l, o_ref, l_ref, bo, bl, what or "full")
    return o, l, o_ref, l_ref


# ------------------------------------------------------------ element-by-element, oracle-sized
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("N", [1, 31, 64, 129, 256, 577, 1000])
def test_small_shapes_full_compare(G, oracle, N, d, causal):
    _full(G, oracle, 2, 3, N, d, causal, seed=150 + N, out_dtype=I.FP16 if N % 2 else I.BF16)


@pytest.mark.parametrize("causal", [False, True])
def test_many_tiles_ragged_tail(G, oracle, causal):
    _full(G, oracle, 1, 2, 2309, 128, causal, seed=177, what="ragged")
    _full(G, oracle, 1, 2, 1531, 64, causal, seed=178, out_dtype=I.BF16, what="ragged")


def test_config_f1(G, oracle):
    w = I.FP8_WORKLOADS["f1"]
    _full(G, oracle, w.B, w.H, w.N, w.d, w.causal, w.seed, what="f1")


# ------------------------------------------------------------ the full-size workloads, sampled rows
@pytest.mark.parametrize("name", ["f3", "f4", "f5"])
def test_fp8_workloads_sampled_rows(G, oracle, name):
    w = I.FP8_WORKLOADS[name]
    print("config %s: B%d H%d N%d d%d causal%d peaky%d" % (name, w.B, w.H, w.N, w.d, w.causal, w.peaky), flush=True)
    q, k, v = I.make_workload(w)
    always = [(0, 0, 0), (w.B - 1, w.H - 1, w.N - 1), (0, 0, w.N // 2), (w.B - 1, 0, 1)]
    rows = I.sample_rows(w.B, w.H, w.N, 96, seed=w.seed + 7, always=always)
    o_ref, l_ref, p = oracle.attn_ref_rows(q, k, v, E4M3, rows, w.scale, w.causal, return_p=True)
    o, l = G.run_gpu_fp8(q, k, v, I.FP16, w.scale, w.causal)
    assert np.isfinite(o).all() and np.isfinite(l).all()
    idx = np.asarray(rows)
    og, lg = o[idx[:, 0], idx[:, 1], idx[:, 2]], l[idx[:, 0], idx[:, 1], idx[:, 2]]
    bo = np.empty_like(o_ref)
    bl = np.empty_like(l_ref)
    for r, (b, h, _) in enumerate(rows):
        bor, blr = G.fp8_bounds(p[r:r + 1], G.e4m3_to_f64(v[b, h]), o_ref[r:r + 1], I.FP16)
        bo[r], bl[r] = bor[0], blr[0]
    G.check_fp8(og, lg, o_ref, l_ref, bo, bl, name)
    if not w.peaky:
        # thousands of keys per row: the rounding errors of P average out and the 16-bit tolerances hold
        G.check(og, lg, o_ref, l_ref, name + " (16-bit tolerances)")


# ------------------------------------------------------------ properties that hold at any size
def test_f4_properties(G, oracle):
    """Full sequence length, two heads: O stays inside the convex hull of the V rows (it is normalised by
    the sum of the rounded probabilities), and splitting the keys into two halves and merging the two
    (O, LSE) pairs by their LSE reproduces the one-shot result -- the identity a key-sharded run relies on."""
    w = I.FP8_WORKLOADS["f4"]
    N, d = w.N, w.d
    q, k, v = I.make_qkv(1, 2, N, d, E4M3, w.seed)
    o, l = G.run_gpu_fp8(q, k, v, I.FP16, w.scale, False)
    vf = G.e4m3_to_f64(v)
    assert np.all(o.max(axis=2) <= vf.max(axis=2) + 1e-3) and np.all(o.min(axis=2) >= vf.min(axis=2) - 1e-3)
    h = N // 2
    # queries 0 .. h-1 against each half of the keys (the kernel takes N queries = N keys, so run the
    # halves as sequences of their own with the first h queries)
    o1, l1 = G.run_gpu_fp8(np.ascontiguousarray(q[:, :, :h]), np.ascontiguousarray(k[:, :, :h]), np.ascontiguousarray(v[:, :, :h]), I.FP16, w.scale, False)
    o2, l2 = G.run_gpu_fp8(np.ascontiguousarray(q[:, :, :h]), np.ascontiguousarray(k[:, :, h:]), np.ascontiguousarray(v[:, :, h:]), I.FP16, w.scale, False)
    lm = np.logaddexp(l1, l2)
    om = np.exp(l1 - lm)[..., None] * o1 + np.exp(l2 - lm)[..., None] * o2
    # both sides carry independent E4M3 rounding of ~8000 probabilities per row: a few 1e-3
    assert np.abs(om - o[:, :, :h]).max() < 1e-2 and np.abs(om - o[:, :, :h]).mean() < 1e-3
    assert np.abs(lm - l[:, :, :h]).max() < 5e-3
    # ... and against the oracle on a few of those rows
    rows = [(0, 0, 0), (0, 1, h - 1), (0, 0, 1234), (0, 1, 4321)]
    o_ref, l_ref = oracle.attn_ref_rows(q, k, v, E4M3, rows, w.scale, False)
    idx = np.asarray(rows)
    assert np.abs(om[idx[:, 0], idx[:, 1], idx[:, 2]] - o_ref).max() < 1e-2
    assert np.abs(lm[idx[:, 0], idx[:, 1], idx[:, 2]] - l_ref).max() < 5e-3


def test_single_head_and_other_stream(G, oracle):
    """B*H = 1 (four workgroups), launched on a stream of its own."""
    import torch
    from paper_2510_14719_amd import binding
    B, H, N, d = 1, 1, 1000, 128
    q, k, v = I.make_qkv(B, H, N, d, E4M3, 199)
    o_ref, l_ref, p = oracle.attn_ref(q, k, v, E4M3, 0.1, True, return_p=True)
    dq, dk, dv = (torch.from_numpy(x).cuda() for x in (q, k, v))
    o = torch.empty((B, H, N, d), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    binding.attn_fwd_fp8(dq, dk, dv, o, lse, B, H, N, d, 0.1, True, stream=st)
    st.synchronize()
    bo, bl = G.fp8_bounds(p, G.e4m3_to_f64(v), o_ref, I.BF16)
    G.check_fp8(o.double().cpu().numpy(), lse.double().cpu().numpy(), o_ref, l_ref, bo, bl, "single head, own stream")


# ------------------------------------------------------------ exact and degenerate cases
@pytest.mark.parametrize("causal", [False, True])
def test_zero_q_gives_running_mean(G, oracle, causal):
    # all probabilities are equal: they round to the same E4M3 value and O is the exact mean
    B, H, N, d = 1, 2, 300, 128
    _, k, v = I.make_qkv(B, H, N, d, E4M3, 191)
    q = np.zeros_like(k)
    o_ref, l_ref = oracle.attn_ref(q, k, v, E4M3, 0.125, causal)
    o, l = G.run_gpu_fp8(q, k, v, I.FP16, 0.125, causal)
    G.check(o, l, o_ref, l_ref, "zero-q", tol_o_max=2e-3, tol_o_mean=3e-4, tol_lse=1e-4)


def test_constant_v_rows_come_back_exactly(G):
    # O is normalised by the sum of the rounded probabilities: a convex combination of equal rows is that row
    B, H, N, d = 1, 2, 700, 128
    q, k, _ = I.make_qkv(B, H, N, d, E4M3, 192)
    row = I.f32_to_e4m3_bits(np.linspace(-3, 3, d).astype(np.float32))
    v = np.ascontiguousarray(np.broadcast_to(row, (B, H, N, d)))
    o, _ = G.run_gpu_fp8(q, k, v, I.FP16, 0.09, True)
    want = G.e4m3_to_f64(row)
    assert np.abs(o - want).max() <= 2.0 ** -10 * 3.0


def test_one_hot_keys_select_value_rows(G, oracle):
    # key j = 16 e_j, query i = 16 e_pi(i): the winning score is 256*scale = 32 above all others
    N, d = 128, 128
    rng = np.random.Generator(np.random.Philox(193))
    perm = rng.permutation(N)
    eye = np.eye(N, d, dtype=np.float32) * 16.0
    k = I.f32_to_e4m3_bits(eye)[None, None]
    q = I.f32_to_e4m3_bits(eye[perm])[None, None]
    v = I.normal_bits((1, 1, N, d), E4M3, 194)
    o, l = G.run_gpu_fp8(q, k, v, I.FP16, 0.125, False)
    vf = G.e4m3_to_f64(v)
    assert np.abs(o[0, 0] - vf[0, 0, perm]).max() < 1e-6
    assert np.abs(l[0, 0] - 32.0).max() < 1e-4


def test_large_scores_exercise_rescaling(G, oracle):
    # keys whose norm grows along the sequence: the row maximum keeps moving, by more than 2^8 at a time
    B, H, N, d = 1, 2, 640, 128
    rng = np.random.Generator(np.random.Philox(195))
    kf = rng.standard_normal((B, H, N, d), dtype=np.float32) * np.linspace(0.2, 6.0, N, dtype=np.float32)[None, None, :, None]
    q = I.normal_bits((B, H, N, d), E4M3, 196, std=2.0)
    k = I.f32_to_e4m3_bits(kf)
    v = I.normal_bits((B, H, N, d), E4M3, 197)
    for causal in (False, True):
        _full(G, oracle, B, H, N, d, causal, seed=0, scale=0.3, what="large-scores", qkv=(q, k, v))


def test_repeat_runs_are_bit_identical(G):
    q, k, v = I.make_qkv(1, 3, 900, 128, E4M3, 198)
    o1, l1 = G.run_gpu_fp8(q, k, v, I.BF16, 0.1, True)
    o2, l2 = G.run_gpu_fp8(q, k, v, I.BF16, 0.1, True)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


def test_argument_errors_on_device_pointers(G):
    import torch
    from paper_2510_14719_amd import binding
    q = torch.zeros(1 * 1 * 64 * 128, dtype=torch.uint8, device="cuda")
    o = torch.zeros(1 * 1 * 64 * 128, dtype=torch.float16, device="cuda")
    lse = torch.zeros(64, dtype=torch.float32, device="cuda")
    assert binding.attn_fwd_fp8_raw(q, q, q, o, lse, 1, 1, 64, 96, 0.1, 0, None, 0) == -2
    assert binding.attn_fwd_fp8_raw(q, q, q, o, lse, 1, 1, 64, 128, float("nan"), 0, None, 0) == -3
    assert binding.attn_fwd_fp8_raw(q, q, q, q.view(torch.float16), lse, 1, 1, 32, 128, 0.1, 0, None, 0) == -7
    with pytest.raises(binding.AttnFwdError):
        binding.attn_fwd_fp8(q, q, q, o, lse, 1, 1, 64, 128, -1.0, False)

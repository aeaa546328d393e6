"""Parity of the HIP path (through the C ABI) with the fp64 CPU oracle.

Tolerances are the benchmark spec's: O max-abs 2e-2, mean-abs 2e-3; LSE max-abs 1e-2.
"""
import math

import numpy as np
import pytest

from paper_2510_14719_amd import inputs as I

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import torch
    assert torch.cuda.is_available(), "the gpu tests need a GPU"
    from tests import gpu_util
    from paper_2510_14719_amd import binding
    binding.load_library()   # fails loudly if the extension was not built
    return gpu_util


def _full(G, oracle, B, H, N, d, dtype, causal, seed, scale=None, peaky=False, what=""):
    q, k, v = I.make_qkv(B, H, N, d, dtype, seed, peaky=peaky)
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    print("case %s B%d H%d N%d d%d dtype%d causal%d seed%d" % (what, B, H, N, d, dtype, causal, seed), flush=True)
    o_ref, l_ref = oracle.attn_ref(q, k, v, dtype, scale, causal)
    o, l = G.run_gpu(q, k, v, dtype, scale, causal)
    G.check(o, l, o_ref, l_ref, what or "full")


# ------------------------------------------------------------ element-by-element, oracle-sized
@pytest.mark.parametrize("dtype", [I.FP16, I.BF16])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("N", [1, 31, 64, 129, 256, 577, 1000])
def test_small_shapes_full_compare(G, oracle, N, d, causal, dtype):
    _full(G, oracle, 2, 3, N, d, dtype, causal, seed=50 + N)


@pytest.mark.parametrize("causal,dtype", [(False, I.FP16), (True, I.BF16)])
def test_more_tiles_than_resident_workgroups(G, oracle, causal, dtype):
    # 650 query tiles at d = 128: a persistent launch walks up to three rounds of its tile schedule,
    # the last one partial, each workgroup switching head and query tile between rounds
    _full(G, oracle, 5, 26, 1100, 128, dtype, causal, seed=77, what="multi-round")


def test_config_c1(G, oracle):
    w = I.WORKLOADS["c1"]
    _full(G, oracle, w.B, w.H, w.N, w.d, w.dtype, w.causal, w.seed, what="c1")


@pytest.mark.parametrize("causal", [False, True])
def test_many_tiles_ragged_tail(G, oracle, causal):
    # several query tiles, many K/V tiles, and a tail that is not a multiple of any tile size
    _full(G, oracle, 1, 2, 2309, 128, I.FP16, causal, seed=77, what="ragged")
    _full(G, oracle, 1, 2, 1531, 64, I.BF16, causal, seed=78, what="ragged")


# ------------------------------------------------------------ the benchmark configurations, sampled rows
def _sampled(G, oracle, name, n_rows):
    w = I.WORKLOADS[name]
    print("config %s: B%d H%d N%d d%d dtype%d causal%d peaky%d" % (name, w.B, w.H, w.N, w.d, w.dtype, w.causal, w.peaky), flush=True)
    q, k, v = I.make_workload(w)
    always = [(0, 0, 0), (w.B - 1, w.H - 1, w.N - 1), (0, 0, w.N // 2), (w.B - 1, 0, 1)]
    rows = I.sample_rows(w.B, w.H, w.N, n_rows, seed=w.seed + 7, always=always)
    o_ref, l_ref = oracle.attn_ref_rows(q, k, v, w.dtype, rows, w.scale, w.causal)
    o, l = G.run_gpu(q, k, v, w.dtype, w.scale, w.causal)
    assert np.isfinite(o).all() and np.isfinite(l).all()
    idx = np.asarray(rows)
    G.check(o[idx[:, 0], idx[:, 1], idx[:, 2]], l[idx[:, 0], idx[:, 1], idx[:, 2]], o_ref, l_ref, name)
    return q, k, v, o, l


@pytest.mark.parametrize("name", ["c2", "c2_causal", "c3", "c4", "c5"])
def test_benchmark_configs_sampled_rows(G, oracle, name):
    _sampled(G, oracle, name, 192)


# ------------------------------------------------------------ the full-size configurations, whole heads
@pytest.mark.parametrize("name", ["c2", "c2_causal", "c3", "c4", "c5"])
def test_whole_heads_of_the_large_configs(G, oracle, name):
    """Full size, the launch configuration ``bench.py`` times: every element of O and LSE was written (the buffers
    start out as NaN), and the first and the last (batch, head) agree with the oracle element by element."""
    w = I.WORKLOADS[name]
    print("config %s whole heads: B%d H%d N%d d%d dtype%d causal%d peaky%d" % (name, w.B, w.H, w.N, w.d, w.dtype, w.causal, w.peaky), flush=True)
    q, k, v = I.make_workload(w)
    o, l = G.run_gpu(q, k, v, w.dtype, w.scale, w.causal)
    assert np.isfinite(o).all() and np.isfinite(l).all(), "an element of O or LSE was never written"
    for (b, h) in [(0, 0), (w.B - 1, w.H - 1)]:
        sl = (slice(b, b + 1), slice(h, h + 1))
        o_ref, l_ref = oracle.attn_ref(np.ascontiguousarray(q[sl]), np.ascontiguousarray(k[sl]), np.ascontiguousarray(v[sl]),
                                       w.dtype, w.scale, w.causal)
        G.check(o[sl], l[sl], o_ref, l_ref, "%s head (%d,%d)" % (name, b, h))


# ------------------------------------------------------------ properties that hold at any size
def test_c4_properties(G):
    """Non-causal: permuting K and V rows together leaves O and LSE unchanged (up to rounding order)."""
    w = I.WORKLOADS["c4"]
    q, k, v = I.make_qkv(1, 2, w.N, w.d, w.dtype, w.seed)
    o1, l1 = G.run_gpu(q, k, v, w.dtype, w.scale, False)
    perm = np.random.Generator(np.random.Philox(3)).permutation(w.N)
    o2, l2 = G.run_gpu(q, np.ascontiguousarray(k[:, :, perm]), np.ascontiguousarray(v[:, :, perm]), w.dtype, w.scale, False)
    assert np.abs(o1 - o2).max() < 5e-3
    assert np.abs(l1 - l2).max() < 1e-3
    # |O| is a convex combination of V rows
    vf = G.bits_to_f64(G.to_device_bits(v), w.dtype)
    assert np.all(o1.max(axis=2) <= vf.max(axis=2) + 1e-2) and np.all(o1.min(axis=2) >= vf.min(axis=2) - 1e-2)


# ------------------------------------------------------------ degenerate and extreme inputs
@pytest.mark.parametrize("causal", [False, True])
def test_zero_q_gives_running_mean(G, oracle, causal):
    B, H, N, d = 1, 2, 300, 64
    _, k, v = I.make_qkv(B, H, N, d, I.FP16, 91)
    q = np.zeros_like(k)
    o_ref, l_ref = oracle.attn_ref(q, k, v, I.FP16, 0.125, causal)
    o, l = G.run_gpu(q, k, v, I.FP16, 0.125, causal)
    G.check(o, l, o_ref, l_ref, "zero-q", tol_lse=1e-4)


@pytest.mark.parametrize("dtype", [I.FP16, I.BF16])
def test_large_scores_exercise_rescaling(G, oracle, dtype):
    # scores with |s| up to ~60 and a maximum that keeps moving along the key axis
    B, H, N, d = 1, 2, 700, 128
    q = I.normal_bits((B, H, N, d), dtype, 92, std=2.0)
    rng = np.random.Generator(np.random.Philox(93))
    kf = rng.standard_normal((B, H, N, d), dtype=np.float32) * (0.5 + 2.5 * np.arange(N, dtype=np.float32)[None, None, :, None] / N)
    k = I.to_bits(kf, dtype)
    v = I.normal_bits((B, H, N, d), dtype, 94)
    scale = 1.0 / math.sqrt(d)
    o_ref, l_ref = oracle.attn_ref(q, k, v, dtype, scale, False)
    o, l = G.run_gpu(q, k, v, dtype, scale, False)
    # near one-hot rows: O inherits the 16-bit rounding of P and of the output, |O| up to ~4
    G.check(o, l, o_ref, l_ref, "large-scores", tol_o_max=4e-2 if dtype == I.BF16 else 2e-2, tol_lse=2e-2)


def test_score_shift_moves_lse_only(G):
    B, H, N, d = 1, 1, 512, 64
    scale, c = 0.125, 24.0
    rng = np.random.Generator(np.random.Philox(95))
    qf = rng.standard_normal((B, H, N, d), dtype=np.float32)
    kf = rng.standard_normal((B, H, N, d), dtype=np.float32)
    qf[..., d - 1] = 0.0
    kf[..., d - 1] = 0.0
    v = I.normal_bits((B, H, N, d), I.FP16, 96)
    o0, l0 = G.run_gpu(I.to_bits(qf, I.FP16), I.to_bits(kf, I.FP16), v, I.FP16, scale, False)
    qf[..., d - 1] = 1.0
    kf[..., d - 1] = c / scale
    o1, l1 = G.run_gpu(I.to_bits(qf, I.FP16), I.to_bits(kf, I.FP16), v, I.FP16, scale, False)
    assert np.abs(o0 - o1).max() < 2e-3
    assert np.abs(l1 - l0 - c).max() < 1e-3


def test_repeat_runs_are_bit_identical(G):
    q, k, v = I.make_qkv(2, 4, 777, 128, I.BF16, 97)
    o0, l0 = G.run_gpu(q, k, v, I.BF16, 0.09, True)
    for _ in range(5):
        o, l = G.run_gpu(q, k, v, I.BF16, 0.09, True)
        assert np.array_equal(o, o0) and np.array_equal(l, l0)


def test_non_default_stream(G, oracle):
    import torch
    q, k, v = I.make_qkv(1, 2, 200, 64, I.FP16, 98)
    o_ref, l_ref = oracle.attn_ref(q, k, v, I.FP16, 0.125, True)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        o, l = G.run_gpu(q, k, v, I.FP16, 0.125, True)
    G.check(o, l, o_ref, l_ref, "side-stream")


def test_argument_errors_on_device_pointers(G):
    import torch
    from paper_2510_14719_amd import binding
    t = torch.zeros(1 * 1 * 64 * 64 + 64, dtype=torch.float16, device="cuda")
    l = torch.zeros(64, dtype=torch.float32, device="cuda")
    o = torch.zeros_like(t)
    assert binding.attn_fwd_raw(t, t, t, o, l, 1, 1, 64, 64, 0.125, 0, None, 0) == 0
    assert binding.attn_fwd_raw(t, t, t, o, l, 1, 1, 64, 96, 0.125, 0, None, 0) == -2
    assert binding.attn_fwd_raw(t, t, t, o, l, 1, 1, 64, 64, -1.0, 0, None, 0) == -3
    assert binding.attn_fwd_raw(t[1:], t, t, o, l, 1, 1, 64, 64, 0.125, 0, None, 0) == -4
    assert binding.attn_fwd_raw(t, t, t, t, l, 1, 1, 64, 64, 0.125, 0, None, 0) == -7
    torch.cuda.synchronize()

"""The seeded input generator: rounding to 16 bit and the peaky-K recipe."""
import numpy as np
import torch

from paper_2510_14719_amd import inputs as I


def test_bf16_rounding_matches_torch():
    x = np.random.Generator(np.random.Philox(1)).standard_normal(100000, dtype=np.float32) * 37.0
    x[:8] = [0.0, -0.0, 1.0, 1.00390625, 1.01171875, -3.0e-39, 65504.0, 3.3895e38]
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(I.f32_to_bf16_bits(x), want)


def test_fp16_rounding_matches_torch():
    x = np.random.Generator(np.random.Philox(2)).standard_normal(100000, dtype=np.float32) * 5.0
    want = torch.from_numpy(x).to(torch.float16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(I.f32_to_f16_bits(x), want)


def test_same_seed_same_bits_and_peaky_rows():
    a = I.make_qkv(1, 2, 200, 8, I.BF16, seed=7, peaky=True)
    b = I.make_qkv(1, 2, 200, 8, I.BF16, seed=7, peaky=True)
    c = I.make_qkv(1, 2, 200, 8, I.BF16, seed=7, peaky=False)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    assert np.array_equal(a[0], c[0]) and np.array_equal(a[2], c[2])
    changed = (a[1] != c[1]).any(axis=-1)
    assert changed.sum(axis=-1).tolist() == [[10, 10]]  # floor(0.05 * 200) rows per head


def test_workload_table_matches_the_benchmark_definition():
    w = I.WORKLOADS
    assert (w["c4"].B, w["c4"].H, w["c4"].N, w["c4"].d, w["c4"].dtype, w["c4"].causal) == (1, 16, 16384, 128, I.FP16, False)
    assert abs(w["c4"].flops - 4 * 16 * 16384 ** 2 * 128) < 1
    assert abs(w["c5"].flops - 4 * 2 * 32 * 8192 ** 2 * 128 / 2) < 1
    assert w["c2"].scale == 0.125

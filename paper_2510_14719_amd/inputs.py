"""Seeded synthetic inputs for the attention-forward workloads.

This module holds none of the method's arithmetic: it draws random numbers,
rounds them to their storage type and returns raw bit patterns (``uint16`` for
fp16 and bf16, ``uint8`` for the 8-bit float E4M3), so the CPU oracle and the
GPU library are fed identical bits.  It is the only module
both sides' tests import.

The paper's attention sweep (Section 5.4: batch 4, head dimension 128, sequence
lengths 1024..16384, causal and non-causal, fp16) uses no dataset; attention
throughput does not depend on the values, so i.i.d. N(0,1) tensors of the same
shapes stand in for it.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

FP16 = 0
BF16 = 1
E4M3 = 2     # OCP 8-bit float: 1 sign, 4 exponent (bias 7), 3 fraction bits, largest finite 448, no infinities


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    N: int
    d: int
    dtype: int          # FP16, BF16 or E4M3 (element type of Q, K, V)
    causal: bool
    peaky: bool = False  # 5 % of the K rows of every head multiplied by 8
    seed: int = 0

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.d))

    @property
    def flops(self) -> float:
        """Credited work: 4*B*H*N^2*d, halved when causal."""
        f = 4.0 * self.B * self.H * float(self.N) ** 2 * self.d
        return f / 2 if self.causal else f


# The five configurations of the benchmark definition (C2 in both variants).
WORKLOADS = {
    "c1": Workload("c1", 1, 2, 128, 64, FP16, False, seed=1000),
    "c2": Workload("c2", 16, 16, 1024, 64, FP16, False, seed=2000),
    "c2_causal": Workload("c2_causal", 16, 16, 1024, 64, FP16, True, seed=2000),
    "c3": Workload("c3", 4, 16, 4096, 128, BF16, False, seed=3000),
    "c4": Workload("c4", 1, 16, 16384, 128, FP16, False, seed=4000),
    "c5": Workload("c5", 2, 32, 8192, 128, BF16, True, peaky=True, seed=5000),
}

# The same shapes in the paper's second attention precision (Section 5.4, "FP8"): Q, K, V drawn as
# above and rounded to E4M3.  c1/c3/c4/c5 with the element type changed and seeds of their own.
FP8_WORKLOADS = {
    "f1": Workload("f1", 1, 2, 128, 128, E4M3, False, seed=11000),
    "f3": Workload("f3", 4, 16, 4096, 128, E4M3, False, seed=13000),
    "f4": Workload("f4", 1, 16, 16384, 128, E4M3, False, seed=14000),
    "f5": Workload("f5", 2, 32, 8192, 128, E4M3, True, peaky=True, seed=15000),
}


def f32_to_f16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> IEEE binary16 bit patterns, round to nearest even."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def f32_to_e4m3_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> E4M3 bit patterns (uint8), round to nearest even, saturating at +-448; NaN -> 0x7f."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    a = np.abs(x).astype(np.float64)
    m, e = np.frexp(a)                               # a = m * 2^e, m in [0.5, 1)
    t = np.rint(m * 16.0)                            # 4 significant bits, ties to even
    e = np.where(t == 16.0, e + 1, e)
    t = np.where(t == 16.0, 8.0, t)
    normal = ((e + 6).astype(np.int64) << 3) | (t.astype(np.int64) - 8)
    sub = np.rint(a * 512.0).astype(np.int64)        # below 2^-6: multiples of 2^-9 (8 = the smallest normal)
    code = np.where(a < 2.0 ** -6, sub, normal)
    code = np.where(a > 448.0, 0x7E, code)           # saturate (464 and above would round past the largest finite)
    code = np.where(np.isnan(a), 0x7F, np.minimum(code, 0x7E))
    return (code | (np.signbit(x).astype(np.int64) << 7)).astype(np.uint8)


def to_bits(x: np.ndarray, dtype: int) -> np.ndarray:
    if dtype == E4M3:
        return f32_to_e4m3_bits(x)
    return f32_to_bf16_bits(x) if dtype == BF16 else f32_to_f16_bits(x)


def normal_bits(shape, dtype: int, seed: int, std: float = 1.0) -> np.ndarray:
    """i.i.d. N(0, std^2) drawn in float32 from Philox(seed), rounded to the storage type."""
    rng = np.random.Generator(np.random.Philox(seed))
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return to_bits(x, dtype)


def make_qkv(B: int, H: int, N: int, d: int, dtype: int, seed: int, peaky: bool = False,
             peak_frac: float = 0.05, peak_gain: float = 8.0):
    """Q, K, V as ``[B,H,N,d]`` bit patterns (uint16, or uint8 for E4M3); seeds ``seed, seed+1, seed+2``.

    With ``peaky`` a fixed seeded choice of ``floor(peak_frac*N)`` distinct key
    rows of every (b, h) is multiplied by ``peak_gain`` in float32 before the
    rounding, which makes the softmax rows close to one-hot.
    """
    shape = (B, H, N, d)
    q = normal_bits(shape, dtype, seed)
    v = normal_bits(shape, dtype, seed + 2)
    rng = np.random.Generator(np.random.Philox(seed + 1))
    kf = rng.standard_normal(size=shape, dtype=np.float32)
    if peaky:
        n_peak = int(np.floor(peak_frac * N))
        for b in range(B):
            for h in range(H):
                idx = rng.permutation(N)[:n_peak]
                kf[b, h, idx, :] *= np.float32(peak_gain)
    k = to_bits(kf, dtype)
    return q, k, v


def make_workload(w: Workload):
    return make_qkv(w.B, w.H, w.N, w.d, w.dtype, w.seed, peaky=w.peaky)


def sample_rows(B: int, H: int, N: int, n: int, seed: int, always=()):
    """``n`` seeded (b, h, i) triples plus the fixed ones in ``always`` (deduplicated)."""
    rng = np.random.Generator(np.random.Philox(seed))
    rows = {tuple(int(x) for x in r) for r in always}
    while len(rows) < n + len(always):
        rows.add((int(rng.integers(B)), int(rng.integers(H)), int(rng.integers(N))))
    return sorted(rows)


# ---------------------------------------------------------------- matrix product workloads
# The paper's matrix-multiplication sweep (Section 5.2): M = N = 8192, K from 256 to 16384, fp16; it
# uses no dataset either, so i.i.d. N(0,1) operands of the same shapes stand in for it.
GEMM_K_SWEEP = (256, 512, 1024, 2048, 4096, 8192, 16384)


def make_ab(M: int, N: int, K: int, dtype: int, seed: int):
    """A ``[M,K]`` and B ``[N,K]`` (both K-contiguous) as bit patterns (uint16, or uint8 for E4M3); seeds ``seed, seed+1``."""
    return normal_bits((M, K), dtype, seed), normal_bits((N, K), dtype, seed + 1)


def sample_entries(M: int, N: int, n: int, seed: int, always=()):
    """``n`` seeded (m, n) pairs plus the fixed ones in ``always`` (deduplicated, sorted)."""
    rng = np.random.Generator(np.random.Philox(seed))
    out = {tuple(int(x) for x in r) for r in always}
    while len(out) < n + len(always):
        out.add((int(rng.integers(M)), int(rng.integers(N))))
    return sorted(out)

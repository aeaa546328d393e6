"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI
binding on uint16 bit patterns and bring O / LSE back as float64."""
import numpy as np
import torch

from paper_2510_14719_amd import binding, inputs as I

# spec tolerances for N(0,1) inputs
TOL_O_MAX = 2e-2
TOL_O_MEAN = 2e-3
TOL_LSE_MAX = 1e-2


def to_device_bits(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).cuda()


def bits_to_f64(t: torch.Tensor, dtype: int) -> np.ndarray:
    """16-bit patterns on the device -> float64 numpy (decoded by torch, not by the oracle)."""
    tt = t.view(torch.bfloat16 if dtype == I.BF16 else torch.float16)
    return tt.to(torch.float64).cpu().numpy()


# Fill patterns of the output buffers before a launch: a NaN in fp16 and in bf16 (0x7FFF) and a float NaN with
# a recognisable payload.  Whatever the kernel does not write stays NaN, so "every element is finite"
# afterwards proves that every element was written; the guard margins must keep the exact patterns.
O_FILL = 0x7FFF
LSE_FILL_BITS = 0x7FC0BEEF


def fresh_outputs(n_o: int, n_l: int, pad: int):
    """(O buffer int16, LSE buffer float32, O view, LSE view): NaN-filled, with ``pad`` guard elements on each side."""
    obuf = torch.full((n_o + 2 * pad,), O_FILL, dtype=torch.int16, device="cuda")
    lbuf = torch.full((n_l + 2 * pad,), LSE_FILL_BITS, dtype=torch.int32, device="cuda").view(torch.float32)
    return obuf, lbuf, obuf[pad:pad + n_o], lbuf[pad:pad + n_l]


def check_guards(obuf, lbuf, n_o: int, n_l: int, pad: int):
    if pad == 0:
        return
    li = lbuf.view(torch.int32)
    assert bool((obuf[:pad] == O_FILL).all()) and bool((obuf[pad + n_o:] == O_FILL).all()), "O guard words overwritten"
    assert bool((li[:pad] == LSE_FILL_BITS).all()) and bool((li[pad + n_l:] == LSE_FILL_BITS).all()), "LSE guard words overwritten"


def run_gpu(q, k, v, dtype, scale, causal, guard=True):
    """Launch the library on [B,H,N,d] uint16 numpy inputs.  Returns (O f64, LSE f64).

    The outputs start out as NaN (an unwritten element stays NaN and fails the finiteness check of
    ``check``); with ``guard`` they sit inside larger buffers whose margins are checked for stray writes."""
    B, H, N, d = q.shape
    dq, dk, dv = to_device_bits(q), to_device_bits(k), to_device_bits(v)
    n_o, n_l = B * H * N * d, B * H * N
    pad = 256 if guard else 0
    obuf, lbuf, o, lse = fresh_outputs(n_o, n_l, pad)
    binding.attn_fwd(dq, dk, dv, o, lse, B, H, N, d, scale, causal, dtype=dtype)
    torch.cuda.synchronize()
    check_guards(obuf, lbuf, n_o, n_l, pad)
    return bits_to_f64(o.reshape(B, H, N, d), dtype), lse.reshape(B, H, N).to(torch.float64).cpu().numpy()


def check(o_gpu, lse_gpu, o_ref, lse_ref, what="", tol_o_max=TOL_O_MAX, tol_o_mean=TOL_O_MEAN, tol_lse=TOL_LSE_MAX):
    assert np.isfinite(o_gpu).all(), what + ": non-finite O"
    assert np.isfinite(lse_gpu).all(), what + ": non-finite LSE"
    eo = np.abs(o_gpu - o_ref)
    el = np.abs(lse_gpu - lse_ref)
    msg = "%s: O max %.3e mean %.3e, LSE max %.3e" % (what, eo.max(), eo.mean(), el.max())
    print(msg, flush=True)
    assert eo.max() <= tol_o_max, msg
    assert eo.mean() <= tol_o_mean, msg
    assert el.max() <= tol_lse, msg


# ---------------------------------------------------------------- 8-bit-float (E4M3) inputs
def run_gpu_fp8(q, k, v, out_dtype, scale, causal):
    """Launch ``attn_fwd_fp8`` on [B,H,N,d] uint8 numpy inputs (E4M3 patterns).  Returns (O f64, LSE f64);
    the outputs sit inside larger buffers whose margins are checked for stray writes."""
    B, H, N, d = q.shape
    dq, dk, dv = (torch.from_numpy(x).cuda() for x in (q, k, v))
    n_o, n_l = B * H * N * d, B * H * N
    pad = 256
    obuf, lbuf, o, lse = fresh_outputs(n_o, n_l, pad)
    binding.attn_fwd_fp8(dq, dk, dv, o, lse, B, H, N, d, scale, causal, out_dtype=out_dtype)
    torch.cuda.synchronize()
    check_guards(obuf, lbuf, n_o, n_l, pad)
    return bits_to_f64(o.reshape(B, H, N, d), out_dtype), lse.reshape(B, H, N).to(torch.float64).cpu().numpy()


def e4m3_to_f64(bits: np.ndarray) -> np.ndarray:
    """E4M3 patterns -> float64 (decoded by torch, not by the oracle)."""
    return torch.from_numpy(np.ascontiguousarray(bits)).view(torch.float8_e4m3fn).to(torch.float64).numpy()


def fp8_bounds(p, vf, o_ref, out_dtype):
    """Worst-case error of the 8-bit path against the exact result, per output element.

    The kernel rounds every unnormalised probability to E4M3 (round to nearest even) before P V
    and normalises by the sum of the rounded values.  With p_j the exact normalised probabilities
    of a row, the weight the kernel gives key j differs from p_j by at most
        E_j = min(p_j, max(2^-4 p_j, 2^-10 max_j p_j))
    (half a unit in the last of 3 fraction bits for normal values; below 2^-6 of the reference,
    which is never smaller than the row maximum, the spacing is 2^-9; a weight that rounds to
    zero is off by itself), so
        |O_gpu - O| <= (sum_j E_j |v_j| + |O| sum_j E_j) / (1 - sum_j E_j)  + rounding of the output
        |LSE_gpu - LSE| <= -ln(1 - sum_j E_j)
    ``p``: [..., n, N] probability rows, ``vf``: [..., N, d] values, ``o_ref``: [..., n, d].
    Returns (bound_O [..., n, d], bound_LSE [..., n]).
    """
    E = np.minimum(p, np.maximum(p * 2.0 ** -4, p.max(axis=-1, keepdims=True) * 2.0 ** -10))
    se = E.sum(axis=-1)
    assert se.max() < 0.5
    u_out = 2.0 ** -8 if out_dtype == I.BF16 else 2.0 ** -11
    bo = ((E @ np.abs(vf)) + np.abs(o_ref) * se[..., None]) / (1.0 - se[..., None])
    bo = bo * 1.01 + np.abs(o_ref) * u_out * 1.01 + 1e-4      # fp32 accumulation, hardware exp2, output rounding
    bl = -np.log1p(-se) * 1.01 + 1e-4
    return bo, bl


def check_fp8(o_gpu, lse_gpu, o_ref, lse_ref, bound_o, bound_l, what=""):
    """Every element inside its worst-case bound; the mean error far inside (rounding errors are
    zero-mean and largely cancel over the keys of a row)."""
    assert np.isfinite(o_gpu).all(), what + ": non-finite O"
    assert np.isfinite(lse_gpu).all(), what + ": non-finite LSE"
    eo, el = np.abs(o_gpu - o_ref), np.abs(lse_gpu - lse_ref)
    msg = "%s: O max %.3e mean %.3e (bound mean %.3e, worst ratio %.2f), LSE max %.3e mean %.3e (worst ratio %.2f)" % (
        what, eo.max(), eo.mean(), bound_o.mean(), (eo / bound_o).max(), el.max(), el.mean(), (el / bound_l).max())
    print(msg, flush=True)
    assert (eo <= bound_o).all(), msg
    assert (el <= bound_l).all(), msg
    assert eo.mean() <= 0.35 * bound_o.mean() + 1e-4, msg
    assert el.mean() <= 0.35 * bound_l.mean() + 1e-4, msg

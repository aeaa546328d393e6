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


def run_gpu(q, k, v, dtype, scale, causal, guard=True):
    """Launch the library on [B,H,N,d] uint16 numpy inputs.  Returns (O f64, LSE f64).

    With ``guard`` the outputs sit inside larger buffers whose margins are checked
    for stray writes."""
    B, H, N, d = q.shape
    dq, dk, dv = to_device_bits(q), to_device_bits(k), to_device_bits(v)
    n_o, n_l = B * H * N * d, B * H * N
    pad = 256 if guard else 0
    obuf = torch.full((n_o + 2 * pad,), 0x7B7B, dtype=torch.int16, device="cuda")
    lbuf = torch.full((n_l + 2 * pad,), -777.0, dtype=torch.float32, device="cuda")
    o = obuf[pad:pad + n_o]
    lse = lbuf[pad:pad + n_l]
    binding.attn_fwd(dq, dk, dv, o, lse, B, H, N, d, scale, causal, dtype=dtype)
    torch.cuda.synchronize()
    if guard:
        assert bool((obuf[:pad] == 0x7B7B).all()) and bool((obuf[pad + n_o:] == 0x7B7B).all()), "O guard words overwritten"
        assert bool((lbuf[:pad] == -777.0).all()) and bool((lbuf[pad + n_l:] == -777.0).all()), "LSE guard words overwritten"
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

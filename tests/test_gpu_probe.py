"""The MFMA-rate probe of the C ABI runs, writes exactly its sink and nothing else."""
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", [0, 1])
def test_mfma_probe_runs_and_stays_in_bounds(dtype):
    import torch
    from paper_2510_14719_amd import binding
    lib = binding.load_library()
    wgs, iters, pad = 24, 50, 128
    n = lib.attn_fwd_mfma_probe_sink_floats(wgs)
    assert n == wgs * 512
    buf = torch.full((n + 2 * pad,), -777.0, dtype=torch.float32, device="cuda")
    sink = buf[pad:pad + n]
    print("mfma probe dtype %d zero operands" % dtype, flush=True)
    flops = binding.mfma_probe(sink, wgs, iters, False, dtype)
    torch.cuda.synchronize()
    assert flops == wgs * 8 * iters * 8 * 32768.0
    assert bool((sink == 0).all())                       # 0 * 0 accumulated: exactly zero
    print("mfma probe dtype %d random operands" % dtype, flush=True)
    binding.mfma_probe(sink, wgs, iters, True, dtype)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(sink).all()) and float(sink.abs().max()) > 0
    assert bool((buf[:pad] == -777.0).all()) and bool((buf[pad + n:] == -777.0).all())
    with pytest.raises(ValueError):
        binding.mfma_probe(sink[:100], wgs, iters, True, dtype)

"""The benchmark-only entry points run and report sane figures (no parity content)."""
import pytest

pytestmark = pytest.mark.gpu


def test_mfma_rate_probe_runs_and_counts_flops():
    import torch
    from paper_2505_13389_amd import vsa
    ops = torch.randn(32768, device="cuda").to(torch.bfloat16)
    sink = torch.full((8 * 256,), float("nan"), device="cuda")
    flops = vsa.vsa_bench_mfma_rate(ops, sink, 8, 10)
    torch.cuda.synchronize()
    assert flops == 8 * 4 * 10 * 32 * 2 * 32 * 32 * 16
    assert torch.isfinite(sink).all()  # every thread wrote its sum


def test_mfma_rate_probe_rejects_bad_arguments():
    import torch
    from paper_2505_13389_amd import vsa
    ops = torch.zeros(32768, device="cuda", dtype=torch.bfloat16)
    sink = torch.zeros(256, device="cuda")
    with pytest.raises(vsa.VsaError):
        vsa.vsa_bench_mfma_rate(ops, sink, 1, 0)

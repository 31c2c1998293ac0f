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


def test_selection_quality_diagnostic_on_planted_inputs(monkeypatch, capsys):
    """Structured inputs: the coarse stage must pick cubes that hold far more of the dense attention
    mass than random cubes do, and no more than the best possible choice."""
    import sys
    from paper_2505_13389_amd import selection_quality
    monkeypatch.setattr(sys, "argv", ["selection_quality", "--workload", "sweep_h8_d64_k32", "--heads", "1"])
    line = selection_quality.main()
    assert line["mass_on_random_cubes"] < 0.5 * line["mass_on_selected_cubes"]
    assert line["mass_on_selected_cubes"] <= line["mass_on_best_cubes"] + 1e-9
    assert abs(line["mass_on_random_cubes"] - line["density"]) < 0.1


def test_topk_sweep_runs_and_scales_with_density(monkeypatch, capsys):
    """The sweep module: one shape, three top-K settings; time must grow with top-K and the
    dense setting must be its own reference."""
    import sys
    from paper_2505_13389_amd import sweep
    monkeypatch.setattr(sys, "argv", ["sweep", "--heads", "8", "--dims", "64", "--topk", "16", "64",
                                      "--steps", "5", "--warmup", "2"])
    rows = sweep.main()
    by_k = {r["topk"]: r for r in rows}
    assert sorted(by_k) == [16, 64, 256]
    assert by_k[256]["fwd_bwd_speedup_vs_dense"] == 1.0
    assert by_k[16]["fwd_bwd_ms"] < by_k[64]["fwd_bwd_ms"] < by_k[256]["fwd_bwd_ms"]
    assert 1.0 < by_k[64]["fwd_bwd_speedup_vs_dense"] <= by_k[64]["ideal_speedup"] * 1.05

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


def test_selection_quality_mass_table_matches_the_oracle():
    """The diagnostic's dense-mass table (torch on the GPU) and the mass it reports for the library's
    own selection, against the oracle's table for the same slice [Sec. 3.5]."""
    import numpy as np
    import sys
    import os
    import torch
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    from helpers import bf16_to_np, grid_of, problem_of, tiled_bits, to_dev
    from oracle import vsa_oracle as orc
    from paper_2505_13389_amd import selection_quality, vsa
    from paper_2505_13389_amd.synth import Workload
    wl = Workload("quality", 1, 1, 7, 14, 15, 64, 6, planted=True)
    bits = tiled_bits(wl, seed=3)
    dev = to_dev(bits)
    g = grid_of(wl)
    valid, _ = orc.valid_mask(g)
    q, k = bf16_to_np(dev["q"][0, 0]), bf16_to_np(dev["k"][0, 0])
    want = orc.block_mass(g, q, k, real="f64")
    got = selection_quality.block_mass(dev["q"][0, 0].float(), dev["k"][0, 0].float(), torch.from_numpy(valid).cuda(),
                                       1.0 / np.sqrt(wl.d)).cpu().numpy()
    assert np.abs(got - want).max() < 1e-5
    buf = vsa.Buffers(problem_of(wl), backward=False)
    buf.forward(dev["q"], dev["k"], dev["v"], dev["gate_c"], dev["gate_f"])
    torch.cuda.synchronize()
    idx = buf.block_idx[0, 0].cpu().numpy()
    ref = orc.forward(g, *(bf16_to_np(dev[n]) for n in ("q", "k", "v", "gate_c", "gate_f")), wl.topk, real="f32")
    assert np.array_equal(idx, ref["block_idx"][0, 0])  # planted inputs: wide gaps, the selection is exact
    on_selected = np.take_along_axis(want, idx.astype(np.int64), axis=1).sum(1).mean()
    on_best = np.sort(want, axis=1)[:, -wl.topk:].sum(1).mean()
    assert on_selected <= on_best + 1e-12 and on_selected > 3 * wl.topk / g.Nc  # far above a random choice


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

"""GPU parity where index lists and in-degrees exceed two 64-entry register chunks: the sweep shape
(B=2, 256 cubes, top-K = 128, planted locality plus two sink cubes that every query cube selects, so that
transposed lists run from a few dozen to 256 entries) at both head dims, and one Wan-14B-shaped head
(1440 cubes, top-K = 180).  The launch is the multi-head one; one (batch, head) slice of it is
compared with the oracle element by element, forward and backward, dK and dV included."""
import numpy as np
import pytest

from helpers import assert_close, bf16_to_np, check_index_sets, grid_of, problem_of, tiled_bits, to_dev
from oracle import vsa_oracle as orc
from paper_2505_13389_amd import synth
from paper_2505_13389_amd.synth import Workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vsa():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2505_13389_amd import vsa as m
    m.lib()
    return m


def slice_to_oracle(dev, b, h):
    return {n: (None if t is None else bf16_to_np(t[b:b + 1, h:h + 1].contiguous())) for n, t in dev.items()}


def compare_slice(vsa, wl, dev, b, h, own_selection_rows_equal=0.0):
    """Full launch on the library's own selection (index-set rule on the slice), then forward and
    backward with the oracle's lists planted into that slice of the launch; returns the oracle lists."""
    import torch
    g = grid_of(wl)
    x = slice_to_oracle(dev, b, h)
    fwd = orc.forward(g, x["q"], x["k"], x["v"], x["gate_c"], x["gate_f"], wl.topk, real="f32", want_sc=True)
    buf = vsa.Buffers(problem_of(wl), backward=True)
    a = (dev["q"], dev["k"], dev["v"], dev["gate_c"], dev["gate_f"])
    buf.forward(*a)
    torch.cuda.synchronize()
    gi = buf.block_idx[b:b + 1, h:h + 1].cpu().numpy()
    differ = check_index_sets(gi, fwd["block_idx"], fwd["sc"])
    assert 1.0 - len(differ) / g.Nc >= own_selection_rows_equal, f"{len(differ)} of {g.Nc} rows differ"
    assert_close(buf.out_coarse[b:b + 1, h:h + 1].cpu().numpy(), fwd["out_coarse"], "out_coarse", 1e-4, 1e-4)

    buf.block_idx[b, h].copy_(torch.from_numpy(fwd["block_idx"][0, 0]))
    buf.forward(*a, indices_given=True)
    buf.backward(*a, dev["dout"], workspace_kept=True)
    torch.cuda.synchronize()
    ref = orc.backward(g, x["q"], x["k"], x["v"], x["gate_c"], x["gate_f"], x["dout"], fwd["block_idx"], wl.topk,
                       real="f32")
    sl = (slice(b, b + 1), slice(h, h + 1))
    assert_close(bf16_to_np(buf.out[sl]), fwd["out"], "out")
    assert np.abs(buf.lse_fine[sl].cpu().numpy() - fwd["lse_fine"]).max() < 2e-3
    for n in ("dq", "dk", "dv", "dgate_c", "dgate_f"):
        assert_close(bf16_to_np(getattr(buf, n)[sl]), ref[n], n)
    return fwd["block_idx"][0, 0]


@pytest.mark.parametrize("d,H,b,h", [(64, 8, 1, 5), (128, 8, 0, 6)])
def test_sweep_shape_topk128_with_sinks(vsa, d, H, b, h):
    wl = Workload(f"sweep_h{H}_d{d}_k128", 2, H, 16, 32, 32, d, 128, planted=True)
    dev = to_dev(tiled_bits(wl, seed=40 + d, sinks=2, sink_gain=0.3))
    idx = compare_slice(vsa, wl, dev, b, h, own_selection_rows_equal=0.9)
    indeg = np.bincount(idx.ravel(), minlength=wl.Nc)
    assert indeg.max() >= 0.9 * wl.Nc, "a sink cube is selected by (nearly) every query cube"
    assert (indeg > 160).sum() >= 8 and (indeg < 100).sum() >= 8, "in-degrees must spread to both sides of 128"


@pytest.mark.parametrize("cube,topk", [((4, 4, 8), 16), ((4, 8, 8), 8)])
def test_mid_shape_with_larger_cubes(vsa, cube, topk):
    """The Mid latent (16x32x32, 12 heads, d=128, 87.5 % sparse) with 128- and 256-token cubes (Sec. 3.2
    tile sizes), as tile_sizes.py times it: one head of the 12-head launch against the oracle."""
    wl = Workload("mid_big_cubes", 1, 12, 16, 32, 32, 128, topk, cube=cube)
    dev = synth.device_iid_inputs(wl, seed=8, tiled_rows=wl.Np)
    compare_slice(vsa, wl, dev, 0, 7, own_selection_rows_equal=0.85)


def test_wan14b_head_topk180_backward(vsa):
    wl = Workload("wan14b_two_heads", 1, 2, 21, 45, 80, 128, 180)
    dev = synth.device_iid_inputs(wl, seed=7, tiled_rows=wl.Np)
    idx = compare_slice(vsa, wl, dev, 0, 1, own_selection_rows_equal=0.9)
    indeg = np.bincount(idx.ravel(), minlength=wl.Nc)
    assert indeg.max() > 192 and indeg.min() < 180, "transposed lists must cross into the fourth register chunk"

"""Mismatched granularity (Sec. 3.2): coarse stage on 64-token cubes, selection and fine stage on tiles of
(1,2,2) cubes, the coarse attention map average-pooled 2x2 on both axes before the top-K.  The
library's tile lists against the oracle's (exact, except where the pooled probabilities of the
differing tiles agree to 1e-4 relative), then forward and backward on the oracle's lists."""
import dataclasses

import numpy as np
import pytest

from helpers import assert_close, bf16_to_np, grid_of, problem_of, tiled_bits, to_dev, widen
from oracle import vsa_oracle as orc
from paper_2505_13389_amd.synth import Workload

pytestmark = pytest.mark.gpu

CASES = {
    "even_d64": Workload("even_d64", 1, 2, 8, 16, 32, 64, 3),
    "ragged_d128": Workload("ragged_d128", 2, 1, 7, 14, 30, 128, 4),
    "planted_d64": Workload("planted_d64", 1, 2, 8, 24, 24, 64, 5, planted=True),
    "all_tiles": Workload("all_tiles", 1, 1, 4, 16, 16, 128, 4),  # top-K = every tile: dense
}


@pytest.fixture(scope="module")
def vsa():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2505_13389_amd import vsa as m
    m.lib()
    return m


@pytest.mark.parametrize("name", list(CASES))
def test_pooled_selection_forward_backward(vsa, name):
    import torch
    wl = CASES[name]
    bits = tiled_bits(wl, seed=21, pad_garbage=True)
    x = widen(bits)
    g = grid_of(wl)
    sel = orc.select_pooled(g, x["q"], x["k"], wl.topk, real="f32")
    K4 = 4 * wl.topk
    fwd = orc.forward(g, x["q"], x["k"], x["v"], x["gate_c"], x["gate_f"], K4, block_idx=sel["cube_idx"], real="f32")
    ref = orc.backward(g, x["q"], x["k"], x["v"], x["gate_c"], x["gate_f"], x["dout"], sel["cube_idx"], K4, real="f32")

    dev = to_dev(bits)
    pb = dataclasses.replace(problem_of(wl), flags=vsa.VSA_FLAG_SELECT_POOLED_2X2)
    buf = vsa.Buffers(pb, backward=True)
    a = (dev["q"], dev["k"], dev["v"], dev["gate_c"], dev["gate_f"])
    buf.forward(*a)
    torch.cuda.synchronize()
    got = buf.block_idx.cpu().numpy()
    assert got.shape == sel["tile_idx"].shape
    Ns = got.shape[2]
    assert (got >= 0).all() and (got < Ns).all() and (np.diff(got, axis=-1) > 0).all()
    differ = np.argwhere((got != sel["tile_idx"]).any(-1))
    for b, h, s in differ:  # near-ties only: the pooled probabilities of the tiles in question agree to 1e-4 relative
        row = sel["pooled"][b, h, s].astype(np.float64)
        p_k = row[sel["tile_idx"][b, h, s]].min()
        for j in set(got[b, h, s]) ^ set(sel["tile_idx"][b, h, s]):
            assert abs(np.log(row[j]) - np.log(p_k)) < 1e-4, (b, h, s, j)
    assert len(differ) <= max(1, Ns // 8)
    if wl.planted:
        assert len(differ) == 0
    assert_close(buf.out_coarse.cpu().numpy(), fwd["out_coarse"], "out_coarse", 1e-4, 1e-4)

    # values on the oracle's selection
    buf.block_idx.copy_(torch.from_numpy(sel["tile_idx"]))
    buf.forward(*a, indices_given=True)
    buf.backward(*a, dev["dout"], workspace_kept=True)
    torch.cuda.synchronize()
    assert_close(bf16_to_np(buf.out), fwd["out"], "out")
    assert np.abs(buf.lse_fine.cpu().numpy() - fwd["lse_fine"]).max() < 2e-3
    for n in ("dq", "dk", "dv", "dgate_c", "dgate_f"):
        assert_close(bf16_to_np(getattr(buf, n)), ref[n], n)
    valid, _ = orc.valid_mask(g)
    for n in ("out", "dq", "dk", "dv"):
        assert not bf16_to_np(getattr(buf, n))[:, :, ~valid].any(), f"{n}: pad rows must be zero"


def test_pooled_selection_needs_even_cube_counts_and_64_token_cubes(vsa):
    odd = dataclasses.replace(vsa.Problem(1, 1, 8, 12, 16, 64, 2), flags=vsa.VSA_FLAG_SELECT_POOLED_2X2)  # 3 cubes along h
    assert vsa.vsa_workspace_bytes(odd, False) == 0
    big = dataclasses.replace(vsa.Problem(1, 1, 8, 16, 32, 64, 2, cube=(4, 4, 8)), flags=vsa.VSA_FLAG_SELECT_POOLED_2X2)
    assert vsa.vsa_workspace_bytes(big, False) == 0
    many = dataclasses.replace(vsa.Problem(1, 1, 8, 16, 16, 64, 9), flags=vsa.VSA_FLAG_SELECT_POOLED_2X2)  # 8 tiles only
    assert vsa.vsa_workspace_bytes(many, False) == 0

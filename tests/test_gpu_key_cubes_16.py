"""The 64 x 16 tiles of the tile-size tables (Sec. 3.2): (4,4,4) query cubes, keys pooled and selected in
the (2,4,2) boxes nested in them.  The library's selection against the oracle's (index-set rule on the
coarse logits), then forward and backward on the oracle's lists, element by element."""
import dataclasses

import numpy as np
import pytest

from helpers import assert_close, bf16_to_np, check_index_sets, grid_of, problem_of, tiled_bits, to_dev, widen
from oracle import vsa_oracle as orc
from paper_2505_13389_amd.synth import Workload

pytestmark = pytest.mark.gpu

KCUBE = (2, 4, 2)
CASES = {
    "even_d64": Workload("even_d64", 1, 2, 8, 16, 16, 64, 12),
    "ragged_d128": Workload("ragged_d128", 2, 1, 7, 14, 30, 128, 10),      # dead key cubes (t = 7 is pad), partial ones
    "odd_k_d128": Workload("odd_k_d128", 1, 2, 5, 10, 22, 128, 7),          # the last tile of a walk holds 3 entries
    "one_entry_d64": Workload("one_entry_d64", 1, 1, 8, 8, 12, 64, 1),
    "planted_d64": Workload("planted_d64", 1, 2, 8, 24, 24, 64, 16, planted=True),
    "long_lists_d64": Workload("long_lists_d64", 1, 1, 8, 32, 32, 64, 150),  # lists beyond two register chunks
    "all_keys_d128": Workload("all_keys_d128", 1, 1, 4, 16, 16, 128, 64),   # top-K = every key cube: dense
}


@pytest.fixture(scope="module")
def vsa():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2505_13389_amd import vsa as m
    m.lib()
    return m


@pytest.mark.parametrize("name", list(CASES))
def test_key_cubes_16_forward_backward(vsa, name):
    import torch
    wl = CASES[name]
    bits = tiled_bits(wl, seed=33, pad_garbage=True)
    x = widen(bits)
    g = grid_of(wl)
    fwd = orc.forward_kq(g, KCUBE, x["q"], x["k"], x["v"], x["gate_c"], x["gate_f"], wl.topk, real="f32", want_sc=True)
    idx = fwd["block_idx"]
    ref = orc.backward_kq(g, KCUBE, x["q"], x["k"], x["v"], x["gate_c"], x["gate_f"], x["dout"], idx, wl.topk, real="f32")

    dev = to_dev(bits)
    pb = dataclasses.replace(problem_of(wl), flags=vsa.VSA_FLAG_KEY_CUBES_16)
    buf = vsa.Buffers(pb, backward=True)
    a = (dev["q"], dev["k"], dev["v"], dev["gate_c"], dev["gate_f"])
    buf.forward(*a)
    torch.cuda.synchronize()
    got = buf.block_idx.cpu().numpy()
    _, kcnt = orc.keycubes(g, KCUBE)
    assert (kcnt[got] > 0).all(), "a dead key cube was selected"
    sc = np.where(np.isfinite(fwd["sc"]), fwd["sc"], -1e30)
    differ = check_index_sets(got, idx, sc)
    assert len(differ) <= max(1, idx.shape[2] // 8)
    if wl.planted:
        assert len(differ) == 0
    assert_close(buf.out_coarse.cpu().numpy(), fwd["out_coarse"], "out_coarse", 1e-4, 1e-4)
    assert np.abs(buf.lse_coarse.cpu().numpy() - fwd["lse_coarse"]).max() < 1e-4

    # values on the oracle's selection
    buf.block_idx.copy_(torch.from_numpy(idx))
    buf.forward(*a, indices_given=True)
    buf.backward(*a, dev["dout"], workspace_kept=True)
    torch.cuda.synchronize()
    assert_close(bf16_to_np(buf.out), fwd["out"], "out")
    assert_close(bf16_to_np(buf.out_fine), fwd["out_fine"], "out_fine")
    assert np.abs(buf.lse_fine.cpu().numpy() - fwd["lse_fine"]).max() < 2e-3
    for n in ("dq", "dk", "dv", "dgate_c", "dgate_f"):
        assert_close(bf16_to_np(getattr(buf, n)), ref[n], n)
    valid, _ = orc.valid_mask(g)
    for n in ("out", "dq", "dk", "dv"):
        assert not bf16_to_np(getattr(buf, n))[:, :, ~valid].any(), f"{n}: pad rows must be zero"
    # a backward that pools again gives the same bits as one on the kept workspace
    dk_kept = buf.dk.clone()
    buf.backward(*a, dev["dout"], workspace_kept=False)
    torch.cuda.synchronize()
    assert torch.equal(buf.dk, dk_kept)


def test_hostile_key_cube_lists_stay_inside_the_buffers(vsa):
    """Caller-supplied lists of key cubes are not validated: entries outside [0, 4 Nc), duplicates and
    disorder give unspecified values, but the calls complete, results are finite and pad rows zero
    (the clamp and skip arithmetic itself is replayed on the host in the ABI tests)."""
    import torch
    wl = CASES["ragged_d128"]
    bits = tiled_bits(wl, seed=8, pad_garbage=True)
    dev = to_dev(bits)
    pb = dataclasses.replace(problem_of(wl), flags=vsa.VSA_FLAG_KEY_CUBES_16)
    buf = vsa.Buffers(pb, backward=True)
    rng = np.random.Generator(np.random.PCG64(6))
    bad = rng.integers(-7, 4 * buf.Nc + 7, size=tuple(buf.block_idx.shape), dtype=np.int64).astype(np.int32)
    bad[0, 0, 0, :] = np.iinfo(np.int32).max
    bad[0, 0, 1, :] = np.iinfo(np.int32).min
    rc, rep = vsa.vsa_host_replay_lists(pb, bad)
    assert rc == 0 and rep["violations"] == 0
    buf.block_idx.copy_(torch.from_numpy(bad))
    a = (dev["q"], dev["k"], dev["v"], dev["gate_c"], dev["gate_f"])
    buf.forward(*a, indices_given=True)
    buf.backward(*a, dev["dout"])
    torch.cuda.synchronize()
    valid, _ = orc.valid_mask(grid_of(wl))
    for n in ("out", "dq", "dk", "dv"):
        t = bf16_to_np(getattr(buf, n))
        assert np.isfinite(t).all(), n
        assert not t[:, :, ~valid].any(), f"{n}: pad rows must be zero"

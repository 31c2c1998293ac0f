"""Seeded random shapes through the whole path: grid, cube shape, head count, head dim and top-K are
drawn from a fixed seed (so the cases are the same on every run), sized so that the CPU oracle
finishes each in about a second.  Forward and backward are compared with the oracle on the oracle's
own index lists; the coarse stage's own lists are checked against the oracle's up to near-ties."""
import numpy as np
import pytest

from helpers import (assert_close, bf16_to_np, check_index_sets, grid_of, problem_of, tiled_bits, to_dev, widen)
from oracle import vsa_oracle as orc
from paper_2505_13389_amd.synth import Workload

pytestmark = pytest.mark.gpu

CUBES = [(4, 4, 4), (2, 4, 8), (1, 8, 8), (8, 4, 2), (2, 2, 16), (4, 8, 2)]


BIG_CUBES = [(4, 4, 8), (2, 8, 8), (8, 4, 4), (4, 8, 8), (8, 8, 4), (2, 8, 16)]  # 128 and 256 tokens


def random_workloads(n, seed=20250513, cubes=CUBES, tag="rnd"):
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    while len(out) < n:
        cube = cubes[rng.integers(len(cubes))]
        # 2..5 cubes per axis, each axis possibly ragged
        dims = [int(c * rng.integers(2, 6) - rng.integers(0, c)) for c in cube]
        pad = [(-d) % c + d for d, c in zip(dims, cube)]
        vol = cube[0] * cube[1] * cube[2]
        nc = pad[0] * pad[1] * pad[2] // vol
        if nc * (vol // 64) > 60:
            continue
        topk = int(rng.integers(1, nc + 1)) if rng.random() < 0.8 else nc
        d = int(rng.choice([64, 128]))
        B, H = (1, 2) if rng.random() < 0.7 else (2, 1)
        out.append(Workload(f"{tag}{len(out)}", B, H, dims[0], dims[1], dims[2], d, topk, cube=cube,
                            planted=bool(rng.random() < 0.3)))
    return out


CASES = random_workloads(12) + random_workloads(6, seed=20250514, cubes=BIG_CUBES, tag="big")


@pytest.fixture(scope="module")
def vsa():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2505_13389_amd import vsa as m
    m.lib()
    return m


@pytest.mark.parametrize("wl", CASES, ids=[f"{w.name}-{w.T}x{w.Hh}x{w.W}-c{'x'.join(map(str, w.cube))}-d{w.d}-k{w.topk}"
                                           for w in CASES])
def test_random_shape_forward_backward(vsa, wl):
    import torch
    with_gate_f = wl.topk % 2 == 0
    bits = tiled_bits(wl, seed=11, with_gate_f=with_gate_f, pad_garbage=True)
    x = widen(bits)
    g = grid_of(wl)
    fwd = orc.forward(g, x["q"], x["k"], x["v"], x["gate_c"], x["gate_f"], wl.topk, real="f32", want_sc=True)
    ref = orc.backward(g, x["q"], x["k"], x["v"], x["gate_c"], x["gate_f"], x["dout"], fwd["block_idx"], wl.topk,
                       real="f32")
    dev = to_dev(bits)
    pb = problem_of(wl)
    buf = vsa.Buffers(pb, backward=True, with_gate_f=with_gate_f)
    # the library's own selection
    buf.forward(dev["q"], dev["k"], dev["v"], dev["gate_c"], dev["gate_f"])
    torch.cuda.synchronize()
    check_index_sets(buf.block_idx.cpu().numpy(), fwd["block_idx"], fwd["sc"])
    # fine stage and backward on the oracle's selection
    buf.block_idx.copy_(torch.from_numpy(fwd["block_idx"]))
    buf.forward(dev["q"], dev["k"], dev["v"], dev["gate_c"], dev["gate_f"], indices_given=True)
    buf.backward(dev["q"], dev["k"], dev["v"], dev["gate_c"], dev["gate_f"], dev["dout"], workspace_kept=True)
    torch.cuda.synchronize()
    assert_close(bf16_to_np(buf.out), fwd["out"], "out")
    for name in ("dq", "dk", "dv", "dgate_c") + (("dgate_f",) if with_gate_f else ()):
        assert_close(bf16_to_np(getattr(buf, name)), ref[name], name)
    valid, _ = orc.valid_mask(g)
    for name in ("out", "dq", "dk", "dv"):
        assert not bf16_to_np(getattr(buf, name))[:, :, ~valid].any(), f"{name}: pad rows must be zero"

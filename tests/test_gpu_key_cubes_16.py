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


def random_cases(n, seed=20250515, tag="rnd16"):
    """Seeded random grids (2..5 cubes per axis, each possibly ragged), head dims, head counts and list
    lengths from 1 to all live key cubes."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = {}
    while len(out) < n:
        dims = [int(4 * rng.integers(2, 6) - rng.integers(0, 4)) for _ in range(3)]
        nc = np.prod([(x + 3) // 4 for x in dims])
        if nc > 60:
            continue
        live = ((dims[0] + 1) // 2) * ((dims[1] + 3) // 4) * ((dims[2] + 1) // 2)
        topk = int(rng.integers(1, live + 1)) if rng.random() < 0.8 else live
        B, H = (1, 2) if rng.random() < 0.7 else (2, 1)
        name = f"{tag}{len(out)}-{dims[0]}x{dims[1]}x{dims[2]}-k{topk}"
        out[name] = Workload(name, B, H, dims[0], dims[1], dims[2], int(rng.choice([64, 128])), topk,
                             planted=bool(rng.random() < 0.3))
    return out


CASES.update(random_cases(8))


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
    with_gate_f = not (name.startswith("rnd16") and wl.topk % 2)   # some of the random cases run without a fine gate
    bits = tiled_bits(wl, seed=33, with_gate_f=with_gate_f, pad_garbage=True)
    x = widen(bits)
    g = grid_of(wl)
    fwd = orc.forward_kq(g, KCUBE, x["q"], x["k"], x["v"], x["gate_c"], x["gate_f"], wl.topk, real="f32", want_sc=True)
    idx = fwd["block_idx"]
    ref = orc.backward_kq(g, KCUBE, x["q"], x["k"], x["v"], x["gate_c"], x["gate_f"], x["dout"], idx, wl.topk, real="f32")

    dev = to_dev(bits)
    pb = dataclasses.replace(problem_of(wl), flags=vsa.VSA_FLAG_KEY_CUBES_16)
    buf = vsa.Buffers(pb, backward=True, with_gate_f=with_gate_f)
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
    for n in ("dq", "dk", "dv", "dgate_c") + (("dgate_f",) if with_gate_f else ()):
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


def _head(dev, b, h):
    return {n: (None if t is None else bf16_to_np(t[b:b + 1, h:h + 1].contiguous())) for n, t in dev.items()}


def test_key_cubes_16_at_the_pretraining_shape_one_head_forward_backward(vsa):
    """16x32x32 latent, 12 heads, d=128, 128 of 1024 key cubes (87.5 % sparse): the 12-head launch, one
    head against the oracle -- selection, forward values where the selections agree, and the backward
    of that head re-run on the oracle's lists."""
    import torch
    from paper_2505_13389_amd import synth
    wl = Workload("mid_key16", 1, 12, 16, 32, 32, 128, 128)
    dev = synth.device_iid_inputs(wl, seed=4, tiled_rows=wl.Np)
    pb = dataclasses.replace(problem_of(wl), flags=vsa.VSA_FLAG_KEY_CUBES_16)
    buf = vsa.Buffers(pb, backward=True)
    a = (dev["q"], dev["k"], dev["v"], dev["gate_c"], dev["gate_f"])
    buf.forward(*a)
    buf.backward(*a, dev["dout"], workspace_kept=True)
    torch.cuda.synchronize()
    h = 7
    one = Workload("slice", 1, 1, wl.T, wl.Hh, wl.W, wl.d, wl.topk)
    g = grid_of(one)
    x = _head(dev, 0, h)
    ref = orc.forward_kq(g, KCUBE, x["q"], x["k"], x["v"], x["gate_c"], x["gate_f"], wl.topk, real="f32", want_sc=True)
    gi = buf.block_idx[:, h:h + 1].cpu().numpy()
    differ = check_index_sets(gi, ref["block_idx"], ref["sc"])
    assert len(differ) <= 12
    same = np.repeat((gi[0, 0] == ref["block_idx"][0, 0]).all(-1), 64)
    assert same.mean() > 0.9
    assert_close(bf16_to_np(buf.out[:, h:h + 1])[0, 0, same], ref["out"][0, 0, same], "out")
    assert np.abs(buf.lse_fine[:, h:h + 1].cpu().numpy()[0, 0, same] - ref["lse_fine"][0, 0, same]).max() < 2e-3
    gref = orc.backward_kq(g, KCUBE, x["q"], x["k"], x["v"], x["gate_c"], x["gate_f"], x["dout"], ref["block_idx"],
                           wl.topk, real="f32")
    for n in ("dq", "dgate_c", "dgate_f"):  # row-local: the 12-head launch itself, where the selections agree
        assert_close(bf16_to_np(getattr(buf, n)[:, h:h + 1])[0, 0, same], gref[n][0, 0, same], n + " (12-head launch)")
    b1 = vsa.Buffers(dataclasses.replace(problem_of(one), flags=vsa.VSA_FLAG_KEY_CUBES_16), backward=True)
    d1 = {n: (None if t is None else t[:, h:h + 1].contiguous()) for n, t in dev.items()}
    b1.block_idx.copy_(torch.from_numpy(ref["block_idx"]))
    a1 = (d1["q"], d1["k"], d1["v"], d1["gate_c"], d1["gate_f"])
    b1.forward(*a1, indices_given=True)
    b1.backward(*a1, d1["dout"])
    torch.cuda.synchronize()
    for n in ("dq", "dk", "dv", "dgate_c", "dgate_f"):
        assert_close(bf16_to_np(getattr(b1, n)), gref[n], n)


def test_key_cubes_16_at_the_wan13b_shape_sampled_cubes(vsa):
    """21x30x52 latent (dead and partial key cubes, 2496 key cubes per head, lists of 312): the 12-head
    forward, sampled query cubes of one head against the oracle."""
    import torch
    from paper_2505_13389_amd import synth
    wl = Workload("wan13b_key16", 1, 12, 21, 30, 52, 128, 312)
    dev = synth.device_iid_inputs(wl, seed=5, tiled_rows=wl.Np)
    pb = dataclasses.replace(problem_of(wl), flags=vsa.VSA_FLAG_KEY_CUBES_16)
    buf = vsa.Buffers(pb, backward=False)
    buf.forward(dev["q"], dev["k"], dev["v"], dev["gate_c"], dev["gate_f"])
    torch.cuda.synchronize()
    h = 3
    g = grid_of(Workload("slice", 1, 1, wl.T, wl.Hh, wl.W, wl.d, wl.topk))
    cubes = np.array([0, 1, 77, 300, 519, 520, 611, 623], dtype=np.int32)  # the last ones lie in the padded t, h slabs
    x = _head(dev, 0, h)
    ref = orc.forward_kq(g, KCUBE, x["q"], x["k"], x["v"], x["gate_c"], x["gate_f"], wl.topk, real="f32", want_sc=True,
                         cubes=cubes)
    gi = buf.block_idx[:, h:h + 1].cpu().numpy()
    _, kcnt = orc.keycubes(g, KCUBE)
    assert (kcnt[gi] > 0).all(), "a dead key cube was selected"
    sc = np.where(np.isfinite(ref["sc"]), ref["sc"], -1e30)
    differ = check_index_sets(gi[:, :, cubes], ref["block_idx"][:, :, cubes], sc[:, :, cubes])
    assert len(differ) <= 2
    assert_close(buf.out_coarse[:, h:h + 1].cpu().numpy()[:, :, cubes], ref["out_coarse"][:, :, cubes], "out_coarse", 1e-4, 1e-4)
    same_c = np.zeros(g.Nc, bool)
    same_c[cubes] = (gi[0, 0, cubes] == ref["block_idx"][0, 0, cubes]).all(-1)
    same = np.repeat(same_c, 64)
    assert same_c[cubes].sum() >= len(cubes) - 2
    assert_close(bf16_to_np(buf.out[:, h:h + 1])[0, 0, same], ref["out"][0, 0, same], "out")
    valid, _ = orc.valid_mask(g)
    assert not bf16_to_np(buf.out)[:, :, ~valid].any()


def test_key_cubes_16_with_the_other_entry_points_and_flags(vsa):
    """The same results, bit for bit, (a) with `out` / `dout` token-major, (b) from the static-scratch
    forward, (c) from three replays of a captured HIP graph with the outputs and the workspace
    poisoned in between."""
    import torch
    wl = CASES["ragged_d128"]
    dev = to_dev(tiled_bits(wl, seed=12, pad_garbage=True))
    a = (dev["q"], dev["k"], dev["v"], dev["gate_c"], dev["gate_f"])
    flag = vsa.VSA_FLAG_KEY_CUBES_16
    ref = vsa.Buffers(dataclasses.replace(problem_of(wl), flags=flag), backward=True)
    ref.forward(*a)
    ref.backward(*a, dev["dout"])
    torch.cuda.synchronize()
    names = ("out", "block_idx", "out_fine", "lse_fine", "out_coarse", "lse_coarse", "dq", "dk", "dv", "dgate_c", "dgate_f")
    same = lambda x, y: torch.equal(x.contiguous().view(torch.uint8), y.contiguous().view(torch.uint8))

    tm = vsa.Buffers(dataclasses.replace(problem_of(wl), flags=flag | vsa.VSA_FLAG_OUT_TOKEN_MAJOR), backward=True)
    tm.forward(*a)
    tm.backward(*a, dev["dout"].permute(0, 2, 1, 3).contiguous())
    torch.cuda.synchronize()
    assert same(tm.out.view(wl.B, tm.Np, wl.H, wl.d).permute(0, 2, 1, 3), ref.out)
    for n in names[1:]:
        assert same(getattr(tm, n), getattr(ref, n)), n

    st = vsa.Buffers(ref.pb, backward=False)
    for n in names[:6]:
        t = getattr(st, n)
        t.fill_(-1) if t.dtype == torch.int32 else t.fill_(float("nan"))
    vsa.vsa_forward_static(ref.pb, *a, st.out, st.block_idx, st.out_fine, st.lse_fine, st.out_coarse, st.lse_coarse)
    torch.cuda.synchronize()
    for n in names[:6]:
        assert same(getattr(st, n), getattr(ref, n)), n

    want = [getattr(ref, n).clone() for n in names]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ref.forward(*a)
        ref.backward(*a, dev["dout"])
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        ref.forward(*a)
        ref.backward(*a, dev["dout"])
    for rep in range(3):
        for n in names:
            t = getattr(ref, n)
            t.fill_(-1) if t.dtype == torch.int32 else t.fill_(float("nan"))
        ref.workspace.fill_(0xFF)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n, w in zip(names, want):
            assert same(getattr(ref, n), w), f"replay {rep}: {n}"

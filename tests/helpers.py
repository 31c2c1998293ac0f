"""Shared plumbing of the GPU parity tests: seeded inputs -> (oracle arrays, device tensors)."""
import numpy as np

from oracle import vsa_oracle as orc
from oracle.vsa_oracle import Grid
from paper_2505_13389_amd import synth

# Tolerances of the parity bar: every output and gradient within max-abs 2e-2 AND rel-L2 1e-2
# of the fp32 oracle; fp32 side outputs (coarse output, log-sum-exps) much tighter.
MAX_ABS = 2e-2
REL_L2 = 1e-2
GAP = 1e-4  # a top-K mismatch is tolerated only where the coarse-logit gap is below this

NAMES = ("q", "k", "v", "gate_c", "gate_f", "dout")


def grid_of(wl):
    return Grid(wl.T, wl.Hh, wl.W, *wl.cube)


def tiled_bits(wl, seed=0, with_gate_f=True, planted=None, pad_garbage=False, sinks=0, sink_gain=1.0):
    """Seeded inputs of a workload as TILED bf16 bit patterns (numpy uint16 [B,H,Np,d]).
    `sinks` > 0 (planted inputs only): that many key cubes attract every query cube."""
    if planted is None:
        planted = wl.planted
    if planted:
        raw = synth.planted_inputs(wl, seed, with_gate_f=with_gate_f, sinks=sinks, sink_gain=sink_gain)
    else:
        assert sinks == 0
        raw = synth.iid_inputs(wl, seed, with_gate_f=with_gate_f)
    g = grid_of(wl)
    out = {}
    for n in NAMES:
        out[n] = None if raw[n] is None else orc.tile_u16(g, raw[n])
    if pad_garbage:
        valid, _ = orc.valid_mask(g)
        rng = np.random.default_rng(99)
        for n in NAMES:
            if out[n] is not None:
                junk = synth.f32_to_bf16_bits(100.0 * rng.standard_normal(out[n][:, :, ~valid].shape, dtype=np.float32))
                out[n][:, :, ~valid] = junk
    return out


def widen(bits):
    """bf16 bits -> float32 arrays for the oracle."""
    return {n: (None if b is None else synth.bf16_bits_to_f32(b)) for n, b in bits.items()}


def to_dev(bits):
    import torch
    return {n: (None if b is None else torch.from_numpy(b.view(np.int16)).cuda().view(torch.bfloat16))
            for n, b in bits.items()}


def bf16_to_np(t):
    import torch
    return synth.bf16_bits_to_f32(t.view(torch.int16).cpu().numpy().view(np.uint16))


def problem_of(wl, topk=None):
    from paper_2505_13389_amd import vsa
    return vsa.problem_of(wl, topk)


def assert_close(got, ref, name, max_abs=MAX_ABS, rel_l2=REL_L2):
    """max-abs and rel-L2 against the oracle.  The absolute bound `max_abs` presumes values of order
    one, as on the benchmark workloads (N(0,1) inputs, lists of 8 or more cubes): the kernels feed
    bf16 operands (2^-9 relative error per term) to the matrix cores and store bf16 (spacing
    2^-7 |x|), so the error of an element scales with the magnitude of the terms it sums, not with
    its own.  For a tensor whose largest reference magnitude M exceeds 2 the bound therefore scales
    with M / 2, and an element is always allowed one spacing of the bf16 output format.  The rel-L2
    bound holds over all elements unchanged."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    diff = np.abs(got - ref)
    err = diff.max() if got.size else 0.0
    big = np.abs(ref).max() if got.size else 0.0
    bound = max_abs * max(1.0, big / 2.0)
    over = (diff - np.maximum(bound, np.abs(ref) * 2.0 ** -7)).max() if got.size else -1.0
    denom = np.sqrt((ref ** 2).sum())
    rel = np.sqrt(((got - ref) ** 2).sum()) / denom if denom > 0 else np.sqrt(((got - ref) ** 2).sum())
    assert over <= 0 and rel <= rel_l2, (f"{name}: max-abs {err:.3e} (<= {bound:.3g}; largest reference magnitude "
                                         f"{big:.3g}), rel-L2 {rel:.3e} (<= {rel_l2})")
    return err, rel


def check_index_sets(gpu_idx, orc_idx, sc, gap=GAP):
    """Top-K parity: per row the sets must be equal, except that an index present on one side
    only is accepted when its coarse logit is within `gap` of the oracle's K-th largest logit
    of that row.  Also checks ascending order and range.  Returns the rows whose sets differ."""
    assert gpu_idx.shape == orc_idx.shape
    Nc = sc.shape[-1]
    assert (gpu_idx >= 0).all() and (gpu_idx < Nc).all()
    assert (np.diff(gpu_idx, axis=-1) > 0).all(), "index lists must be strictly ascending"
    differ = np.argwhere((gpu_idx != orc_idx).any(axis=-1))
    for b, h, c in differ:
        g, o, row = set(gpu_idx[b, h, c]), set(orc_idx[b, h, c]), sc[b, h, c]
        s_k = row[orc_idx[b, h, c]].min()
        for j in (g - o) | (o - g):
            assert abs(row[j] - s_k) < gap, f"row {(b, h, c)}: index {j} differs, logit gap {abs(row[j] - s_k):.3e}"
    return differ

"""vsa_forward_static (the forward on the library's own static scratch, for callers that cannot
allocate) against vsa_forward: same kernels on a different scratch buffer, so every output must
come out bit for bit, on two calls in a row that share the buffer, the second one smaller."""
import pytest

from helpers import problem_of, tiled_bits, to_dev
from paper_2505_13389_amd.synth import WORKLOADS, Workload

pytestmark = pytest.mark.gpu

OUTPUTS = ("out", "block_idx", "out_fine", "lse_fine", "out_coarse", "lse_coarse")


def _both_ways(vsa, wl, seed):
    import torch
    dev = to_dev(tiled_bits(wl, seed=seed, pad_garbage=True))
    pb = problem_of(wl)
    assert vsa.vsa_workspace_bytes(pb, False) <= vsa.lib().vsa_static_scratch_bytes()
    a = (dev["q"], dev["k"], dev["v"], dev["gate_c"], dev["gate_f"])
    ref = vsa.Buffers(pb, backward=False)
    ref.forward(*a)
    got = vsa.Buffers(pb, backward=False)
    for n in OUTPUTS:
        t = getattr(got, n)
        t.fill_(-1) if t.dtype == torch.int32 else t.fill_(float("nan"))
    return ref, got, a, pb


def test_static_scratch_forward_matches_forward_twice_in_a_row():
    import torch
    from paper_2505_13389_amd import vsa
    vsa.lib()
    big = Workload("static_big", 1, 3, 9, 22, 26, 128, 11)     # 126 cubes, ragged on every axis
    small = Workload("static_small", 2, 1, 5, 6, 7, 64, 3)     # 8 cubes: the call after it reuses a dirty buffer
    for wl, seed in ((big, 31), (small, 32)):
        ref, got, a, pb = _both_ways(vsa, wl, seed)
        vsa.vsa_forward_static(pb, *a, got.out, got.block_idx, got.out_fine, got.lse_fine, got.out_coarse,
                               got.lse_coarse)
        torch.cuda.synchronize()
        for n in OUTPUTS:
            assert torch.equal(getattr(got, n).view(torch.uint8), getattr(ref, n).view(torch.uint8)), (wl.name, n)


def test_static_scratch_forward_refuses_what_does_not_fit():
    import torch
    from paper_2505_13389_amd import vsa
    wl = WORKLOADS["wan14b"]  # needs about half a gigabyte of scratch
    pb = problem_of(wl)
    assert vsa.vsa_workspace_bytes(pb, False) > vsa.lib().vsa_static_scratch_bytes()
    x = torch.zeros(64, dtype=torch.bfloat16, device="cuda")  # never touched: the refusal comes first
    with pytest.raises(vsa.VsaError) as e:
        vsa.vsa_forward_static(pb, x, x, x, x, None, x, None, None, None, None, None)
    assert e.value.status == -7

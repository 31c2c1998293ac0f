"""The differentiable PyTorch op (raster token-major tensors in and out; App. B: tile -> attention ->
untile) against the oracle: output and all five gradients through torch.autograd."""
import numpy as np
import pytest

from helpers import assert_close, bf16_to_np, grid_of
from oracle import vsa_oracle as orc
from paper_2505_13389_amd import synth
from paper_2505_13389_amd.synth import Workload

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("wl,with_gate_f", [(Workload("op_a", 1, 2, 8, 16, 16, 64, 8), True),
                                            (Workload("op_b", 2, 3, 7, 14, 30, 128, 6), False)])
def test_autograd_op_matches_the_oracle(wl, with_gate_f):
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    from paper_2505_13389_amd.autograd import video_sparse_attention
    raw = synth.iid_inputs(wl, 41, with_gate_f=with_gate_f)   # raster bf16 bits [B,H,L,d]
    g = grid_of(wl)
    x = {n: (None if b is None else synth.bf16_bits_to_f32(orc.tile_u16(g, b))) for n, b in raw.items()}
    fwd = orc.forward(g, x["q"], x["k"], x["v"], x["gate_c"], x["gate_f"], wl.topk, real="f32")
    ref = orc.backward(g, x["q"], x["k"], x["v"], x["gate_c"], x["gate_f"], x["dout"], fwd["block_idx"], wl.topk, real="f32")

    def dev(bits):  # [B,H,L,d] bits -> token-major bf16 [B,L,H,d]
        t = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
        return t.permute(0, 2, 1, 3).contiguous()

    names = ["q", "k", "v", "gate_c"] + (["gate_f"] if with_gate_f else [])
    t = {n: dev(raw[n]).requires_grad_(True) for n in names}
    out = video_sparse_attention(t["q"], t["k"], t["v"], t["gate_c"], t.get("gate_f"), grid=(wl.T, wl.Hh, wl.W), topk=wl.topk)
    grads = torch.autograd.grad(out, [t[n] for n in names], grad_outputs=dev(raw["dout"]))
    torch.cuda.synchronize()

    def untile(a):  # oracle [B,H,Np,d] float -> raster token-major [B,L,H,d]
        bits = synth.f32_to_bf16_bits(a.astype(np.float32))
        return synth.bf16_bits_to_f32(orc.tile_u16(g, bits, inverse=True)).transpose(0, 2, 1, 3)

    # (both sides go through one more bf16 rounding of the reference here; the bound has room for it)
    assert_close(bf16_to_np(out.detach()), untile(fwd["out"]), "out")
    for n, gr in zip(names, grads):
        key = {"q": "dq", "k": "dk", "v": "dv", "gate_c": "dgate_c", "gate_f": "dgate_f"}[n]
        assert_close(bf16_to_np(gr), untile(ref[key]), key)

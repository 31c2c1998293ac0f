"""Selection-quality diagnostic (Sec. 3.5 asks how much of the dense attention mass the selected
cubes hold): for every query cube, the share of the dense softmax mass of its tokens that falls
on the K key cubes the coarse stage selected, against K random cubes and against the best
possible K cubes.

The selection comes from the HIP library (vsa_forward's block_idx); the dense attention mass is
plain torch arithmetic on the GPU.  It is a measurement aid, not part of the attention path.

    python -m paper_2505_13389_amd.selection_quality [--workload sweep_h8_d64_k32] [--seed 0]
"""
import argparse
import json
import math


def block_mass(q, k, valid, scale, chunk=2048):
    """q, k: fp32 [Np, d] tiled; valid: bool [Np].  Returns [Nc, Nc]: mean over the valid tokens of
    query cube i of the dense softmax mass on key cube j (rows sum to 1)."""
    import torch
    Np = q.shape[0]
    Nc = Np // 64
    out = torch.zeros((Nc, Nc), dtype=torch.float64, device=q.device)
    neg = torch.where(valid, 0.0, float("-inf")).to(torch.float32)
    for r0 in range(0, Np, chunk):
        s = (q[r0:r0 + chunk] @ k.T) * scale + neg[None, :]
        p = torch.softmax(s, dim=-1).to(torch.float64)
        p = p * valid[r0:r0 + chunk, None]
        pm = p.reshape(p.shape[0] // 64, 64, Nc, 64).sum(dim=(1, 3))
        out[r0 // 64:(r0 + chunk) // 64] = pm
    cnt = valid.reshape(Nc, 64).sum(dim=1).clamp(min=1).to(torch.float64)
    return out / cnt[:, None]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="sweep_h8_d64_k32")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--heads", type=int, default=2, help="(batch, head) slices to examine")
    args = ap.parse_args()
    import numpy as np
    import torch
    from . import synth, vsa
    wl = synth.WORKLOADS[args.workload]
    pb = vsa.Problem(wl.B, wl.H, wl.T, wl.Hh, wl.W, wl.d, wl.topk, wl.cube)
    Np, Nc = vsa.vsa_padded_tokens(pb)
    raw = synth.make_inputs(wl, args.seed)
    dev = {}
    for n, b in raw.items():
        src = torch.from_numpy(b.view("int16")).cuda().view(torch.bfloat16)
        dst = torch.empty((wl.B, wl.H, Np, wl.d), dtype=torch.bfloat16, device="cuda")
        vsa.vsa_tile_permute(pb, src, dst)
        dev[n] = dst
    valid_src = torch.ones((wl.B, wl.H, wl.L, wl.d), dtype=torch.bfloat16, device="cuda")
    valid_t = torch.empty((wl.B, wl.H, Np, wl.d), dtype=torch.bfloat16, device="cuda")
    vsa.vsa_tile_permute(pb, valid_src, valid_t)
    valid = valid_t[0, 0, :, 0] > 0
    buf = vsa.Buffers(pb, backward=False)
    buf.forward(dev["q"], dev["k"], dev["v"], dev["gate_c"], dev["gate_f"])
    torch.cuda.synchronize()
    g = torch.Generator(device="cuda")
    g.manual_seed(synth.BASE_SEED + 77 + args.seed)
    scale = 1.0 / math.sqrt(wl.d)
    got, rnd, best = [], [], []
    slices = [(b, h) for b in range(wl.B) for h in range(wl.H)][:args.heads]
    for b, h in slices:
        m = block_mass(dev["q"][b, h].float(), dev["k"][b, h].float(), valid, scale)
        idx = buf.block_idx[b, h].long()
        got.append(m.gather(1, idx).sum(1).mean().item())
        ridx = torch.rand((Nc, Nc), generator=g, device="cuda").argsort(dim=1)[:, :wl.topk]
        rnd.append(m.gather(1, ridx).sum(1).mean().item())
        best.append(m.topk(wl.topk, dim=1).values.sum(1).mean().item())
    line = {"workload": wl.name, "planted": wl.planted, "Nc": Nc, "topk": wl.topk, "slices": len(slices),
            "mass_on_selected_cubes": float(np.mean(got)), "mass_on_random_cubes": float(np.mean(rnd)),
            "mass_on_best_cubes": float(np.mean(best)), "density": wl.topk / Nc}
    print(json.dumps(line))
    return line


if __name__ == "__main__":
    main()

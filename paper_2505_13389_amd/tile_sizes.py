"""Throughput against tile size (the "TFLOPS" column of the tile-size ablation, Sec. 3.2): the same
16x32x32 latent (16384 tokens), 87.5 % tile sparsity, with cubes of 64, 128 and 256 tokens, i.e.
top-K = 32 of 256, 16 of 128 and 8 of 64 cubes, the mismatched setting of that section (coarse
stage on 64-token cubes, fine stage on 256-token tiles, top-K = 8 of 64 tiles on the pooled map) and
its 64 x 16 tiles (64-token query cubes, key cubes of 16 tokens, top-K = 128 of 1024).  Forward and
forward+backward, effective TFLOP/s on the selected blocks.  Synthetic i.i.d. inputs; a measurement aid that calls the library exactly as
the benchmark does.

    python -m paper_2505_13389_amd.tile_sizes [--heads 12] [--dim 128] [--steps 20]
"""
import argparse
import json

# (cube, top-K, flags, key tokens per list entry)
CUBES = [((4, 4, 4), 32, 0, 64), ((4, 4, 8), 16, 0, 128), ((4, 8, 8), 8, 0, 256), ((4, 4, 4), 8, "pooled", 256),
         ((4, 4, 4), 128, "key16", 16)]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--heads", type=int, default=12)
    ap.add_argument("--dim", type=int, default=128)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    args = ap.parse_args()
    import numpy as np
    import torch
    from . import vsa

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        ts = []
        for _ in range(args.steps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            e1.synchronize()
            ts.append(e0.elapsed_time(e1))
        return float(np.median(ts))

    rows = []
    for cube, K, variant, V in CUBES:
        flags = {0: 0, "pooled": vsa.VSA_FLAG_SELECT_POOLED_2X2, "key16": vsa.VSA_FLAG_KEY_CUBES_16}[variant]
        pb = vsa.Problem(1, args.heads, 16, 32, 32, args.dim, K, cube=cube, flags=flags)
        Np, Nc = vsa.vsa_padded_tokens(pb)
        g = torch.Generator(device="cuda")
        g.manual_seed(3)
        shape = (1, args.heads, Np, args.dim)
        q, k, v, do = (torch.randn(shape, generator=g, device="cuda").to(torch.bfloat16) for _ in range(4))
        gc, gf = (torch.rand(shape, generator=g, device="cuda").to(torch.bfloat16) for _ in range(2))
        buf = vsa.Buffers(pb)

        def both():
            buf.forward(q, k, v, gc, gf)
            buf.backward(q, k, v, gc, gf, do, workspace_kept=True)

        tf, tb = timed(lambda: buf.forward(q, k, v, gc, gf)), timed(both)
        fl = 4.0 * Np * K * V * args.dim * args.heads  # V = key tokens per list entry
        line = {"tile": V if variant != "key16" else "64x16", "coarse_cube": list(cube), "tiles": Np // V, "topk": K, "sparsity": 1.0 - K * V / Np, "fwd_ms": round(tf, 4),
                "fwd_bwd_ms": round(tb, 4), "fwd_tflops": round(fl / tf / 1e9, 1),
                "fwd_bwd_tflops": round(3.5 * fl / tb / 1e9, 1)}
        print(json.dumps(line), flush=True)
        rows.append(line)
    return rows


if __name__ == "__main__":
    main()

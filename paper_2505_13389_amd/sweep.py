"""Sparsity sweep (the shape of Fig. 3a/3b and of the kernel-benchmark paragraph of Sec. 3.4): time of
the whole VSA forward and forward+backward against top-K on the sweep shapes (B=2, grid 16x32x32 =
256 cubes, H in {8,16}, d in {64,128}), on planted-locality inputs (queries prefer the 3x3x3
neighbourhood of their cube), with top-K = all cubes as the dense reference of the same code path.

Prints one JSON line per (H, d, top-K) and a closing table.  Synthetic inputs; a measurement aid that
calls the library exactly as the benchmark does.

    python -m paper_2505_13389_amd.sweep [--heads 8 16] [--dims 64 128] [--topk 8 16 32 64 128 256]
"""
import argparse
import json


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--heads", type=int, nargs="+", default=[8, 16])
    ap.add_argument("--dims", type=int, nargs="+", default=[64, 128])
    ap.add_argument("--topk", type=int, nargs="+", default=[8, 16, 32, 64, 128, 256])
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--iid", action="store_true", help="i.i.d. N(0,1) inputs instead of planted locality")
    ap.add_argument("--sinks", type=int, default=0, help="planted inputs: key cubes that every query cube selects")
    ap.add_argument("--sink-gain", type=float, default=1.0)
    args = ap.parse_args()
    import numpy as np
    import torch
    from . import synth, vsa

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
    for H in args.heads:
        for d in args.dims:
            wl = synth.Workload(f"sweep_h{H}_d{d}", 2, H, 16, 32, 32, d, 32, planted=not args.iid)
            raw = (synth.iid_inputs(wl, 0) if args.iid else
                   synth.planted_inputs(wl, 0, sinks=args.sinks, sink_gain=args.sink_gain))
            base = vsa.Problem(wl.B, wl.H, wl.T, wl.Hh, wl.W, wl.d, wl.topk, wl.cube)
            Np, Nc = vsa.vsa_padded_tokens(base)
            dev = {}
            for n, b in raw.items():
                src = torch.from_numpy(b.view("int16")).cuda().view(torch.bfloat16)
                dev[n] = torch.empty((wl.B, wl.H, Np, wl.d), dtype=torch.bfloat16, device="cuda")
                vsa.vsa_tile_permute(base, src, dev[n])
            del raw
            res = {}
            for K in sorted(set(args.topk) | {Nc}):
                if K > Nc:
                    continue
                pb = vsa.Problem(wl.B, wl.H, wl.T, wl.Hh, wl.W, wl.d, K, wl.cube)
                buf = vsa.Buffers(pb)
                a = (dev["q"], dev["k"], dev["v"], dev["gate_c"], dev["gate_f"])

                def fwd():
                    buf.forward(*a)

                def both():
                    buf.forward(*a)
                    buf.backward(*a, dev["dout"], workspace_kept=True)

                res[K] = (timed(fwd), timed(both))
                del buf
            for K, (tf, tb) in res.items():
                fl = 4.0 * Np * K * 64 * wl.d * wl.H * wl.B
                line = {"H": H, "d": d, "Nc": Nc, "topk": K, "sparsity": 1.0 - K / Nc, "planted": wl.planted, "sinks": args.sinks,
                        "fwd_ms": tf, "fwd_bwd_ms": tb, "fwd_tflops": fl / tf / 1e9,
                        "fwd_bwd_tflops": 3.5 * fl / tb / 1e9,
                        "fwd_speedup_vs_dense": res[Nc][0] / tf, "fwd_bwd_speedup_vs_dense": res[Nc][1] / tb,
                        "ideal_speedup": Nc / K}
                print(json.dumps(line), flush=True)
                rows.append(line)
    print(f"{'H':>3} {'d':>4} {'K':>4} {'sparsity':>8} {'fwd ms':>8} {'f+b ms':>8} {'fwd TF/s':>9} {'f+b TF/s':>9} "
          f"{'fwd x':>6} {'f+b x':>6} {'ideal':>6}")
    for r in rows:
        print(f"{r['H']:3d} {r['d']:4d} {r['topk']:4d} {r['sparsity']:8.3f} {r['fwd_ms']:8.3f} {r['fwd_bwd_ms']:8.3f} "
              f"{r['fwd_tflops']:9.1f} {r['fwd_bwd_tflops']:9.1f} {r['fwd_speedup_vs_dense']:6.2f} "
              f"{r['fwd_bwd_speedup_vs_dense']:6.2f} {r['ideal_speedup']:6.1f}")
    return rows


if __name__ == "__main__":
    main()

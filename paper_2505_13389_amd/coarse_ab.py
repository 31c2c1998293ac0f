"""Coarse stage with and without fusion (the comparison of App. D's runtime table, on this chip):
the forward of the named workloads with the coarse stage as three launches (scores = Qc Kc^T into
HBM, softmax + top-K + index list, O_c = P Vc) and as one launch that keeps the score block in LDS
(VSA_FLAG_COARSE_FUSED, up to 256 cubes).  Prints the whole forward time and the per-kernel times
(HIP events around every launch) for both.  A measurement aid; synthetic i.i.d. inputs.

    python -m paper_2505_13389_amd.coarse_ab [tiny mid sweep_h16_d128_k32 ...]
"""
import dataclasses
import json
import sys


def main(names=None):
    import torch
    from . import vsa
    from .synth import WORKLOADS
    rows = []
    for name in names or sys.argv[1:] or ["tiny", "mid"]:
        wl = WORKLOADS[name]
        for fused in (False, True):
            pb = dataclasses.replace(vsa.problem_of(wl),
                                     flags=vsa.VSA_FLAG_COARSE_FUSED if fused else vsa.VSA_FLAG_COARSE_UNFUSED)
            Np, Nc = vsa.vsa_padded_tokens(pb)
            g = torch.Generator(device="cuda")
            g.manual_seed(0)
            shape = (wl.B, wl.H, Np, wl.d)
            q, k, v = (torch.randn(shape, generator=g, device="cuda").to(torch.bfloat16) for _ in range(3))
            gc, gf = (torch.rand(shape, generator=g, device="cuda").to(torch.bfloat16) for _ in range(2))
            buf = vsa.Buffers(pb, backward=False)
            steps = 20
            for _ in range(3):
                buf.forward(q, k, v, gc, gf)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(steps):
                buf.forward(q, k, v, gc, gf)
            e1.record()
            torch.cuda.synchronize()
            whole = e0.elapsed_time(e1) / steps
            vsa.vsa_profile_begin(16 * steps)
            for _ in range(steps):
                buf.forward(q, k, v, gc, gf)
            torch.cuda.synchronize()
            per = {}
            for n, t in vsa.vsa_profile_end():
                per[n] = per.get(n, 0.0) + t / steps
            line = {"workload": name, "Nc": Nc, "coarse": "one launch" if fused else "three launches",
                    "forward_ms": round(whole, 4), "kernel_ms": {n: round(t, 4) for n, t in per.items()},
                    "coarse_share_of_forward": round(per["coarse"] / sum(per.values()), 4)}
            print(json.dumps(line), flush=True)
            rows.append(line)
    return rows


if __name__ == "__main__":
    main()

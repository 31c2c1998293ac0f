#!/usr/bin/env python3
"""Benchmark of the Video Sparse Attention hot path on one MI355X.

One step = vsa_forward + vsa_backward (pooling, coarse attention, top-K, fine block-sparse
attention, gated sum, and the whole backward) on the Wan-1.3B-shaped 480p workload
(valid grid 21x30x52 padded to 24x32x52 = 39936 tokens, 12 heads, d=128, top-K 78 of 624
cubes), inputs resident in HBM in the cube-contiguous layout.  The raster<->tiled
permutation is hoistable out of the layer (App. B listing caption) and is timed separately.

Prints ONE JSON line: effective TFLOP/s counted on the selected 64x64 blocks only
(forward 4*Np*K*64*d*H*B, forward+backward 3.5x, App. C.4), the roofline position of the
dominant kernel, the speedup over the same library's dense path (top-K = all cubes), and the
CPU oracle timed on the host cores on a few heads of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E

# Algorithmic MFMA flops one launch of each fine kernel is credited with, per selected
# (query tile, key tile) pair, in units of 2*64*64*d (one 64x64xd matmul).  Forward: S and PV.
# Backward is 2.5x forward = 5 matmuls (S, dP, dV, dK, dQ); the two-pass backward recomputes S
# and dP in both passes, so each pass is credited half of them: dQ pass 1 + 1, dK/dV pass 2 + 1.
MATMULS = {"fine_fwd": 2.0, "fine_bwd_dq": 2.0, "fine_bwd_dkv": 3.0}
# ... and the matmuls each pass really executes per pair (dQ: S, dP, dQ; dK/dV: S, dP, dV, dK)
EXECUTED = {"fine_fwd": 2.0, "fine_bwd_dq": 3.0, "fine_bwd_dkv": 4.0}
# HBM-side bytes per launch of the fine kernels: measured by rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE)
# in a run of its own and committed with the summaries; this run only replays the figure.
TRAFFIC_FILE = os.path.join("profiles", "traffic_wan1.3b.json")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="wan1.3b")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the other named configurations")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--heads", type=int, default=0, help="override the workload's head count (experiments)")
    return ap.parse_args()


def device_inputs(wl, seed, torch):
    """Seeded inputs drawn on the host in raster order, moved to HBM and tiled by the library."""
    from paper_2505_13389_amd import synth, vsa
    raw = synth.make_inputs(wl, seed)
    pb = vsa.problem_of(wl)
    Np, _ = vsa.vsa_padded_tokens(pb)
    dev = {}
    for n, b in raw.items():
        src = torch.from_numpy(b.view("int16")).cuda().view(torch.bfloat16)
        dst = torch.empty((wl.B, wl.H, Np, wl.d), dtype=torch.bfloat16, device="cuda")
        vsa.vsa_tile_permute(pb, src, dst, inverse=False)
        dev[n] = dst
        dev["raster_" + n] = src
    torch.cuda.synchronize()
    return dev


def time_steps(fn, steps, warmup, torch):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def event_times(fn, n, torch, before=None):
    """n calls of fn, each bracketed by a pair of events on the current stream; ms per call."""
    out = []
    for _ in range(n):
        if before is not None:
            before()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        b.synchronize()
        out.append(a.elapsed_time(b))
    return out


def mfma_rate(torch, vsa):
    """Sustained v_mfma_f32_32x32x16_bf16 rate of this chip on N(0,1) operands, TFLOP/s."""
    g = torch.Generator(device="cuda")
    g.manual_seed(1)
    ops = torch.randn(32768, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    wgs, iters = 1024, 4000
    sink = torch.empty(wgs * 256, device="cuda", dtype=torch.float32)
    fl = vsa.vsa_bench_mfma_rate(ops, sink, wgs, iters)  # warm-up
    torch.cuda.synchronize()
    ms = min(event_times(lambda: vsa.vsa_bench_mfma_rate(ops, sink, wgs, iters), 3, torch))
    return fl / (ms * 1e-3) / 1e12


def hbm_rates(wl, buf, kern, ms_perm):
    tensor = wl.B * wl.H * buf.Np * wl.d * 2           # one tiled bf16 tensor
    raster = wl.B * wl.H * wl.L * wl.d * 2             # one raster bf16 tensor
    pooled = wl.B * wl.H * buf.Nc * wl.d * 4
    rows = wl.B * wl.H * buf.Np
    steps = {"pool": (3 * tensor + 3 * pooled, kern.get("pool")),
             "bwd_pre": (4 * tensor + 3 * tensor + rows * (4 + 8 + 16) + 2 * pooled, kern.get("bwd_pre")),
             "tile_permute_12_tensors": (12 * (tensor + raster), ms_perm)}
    out = {}
    for name, (nbytes, ms_) in steps.items():
        if ms_:
            gbs = nbytes / (ms_ * 1e-3) / 1e9
            out[name] = {"bytes": nbytes, "ms": round(ms_, 4), "GBps": round(gbs, 1), "frac_of_hbm_peak": round(gbs / PEAK_HBM_GBS, 3)}
    return out


def other_configs(torch, vsa, WORKLOADS, Workload, time_steps):
    """The other named configurations, through the same entry points (inputs drawn on the device):
    mid forward+backward, the Wan-14B-shaped forward and forward+backward at top-K 180, and its forward at
    top-K = all 1440 cubes."""
    from paper_2505_13389_amd import synth
    out = {}

    def run(name, wl, backward, steps):
        dev = synth.device_iid_inputs(wl, seed=9, tiled_rows=wl.Np)
        buf = vsa.Buffers(vsa.problem_of(wl), backward=backward)
        a = (dev["q"], dev["k"], dev["v"], dev["gate_c"], dev["gate_f"])

        def step():
            buf.forward(*a)
            if backward:
                buf.backward(*a, dev["dout"], workspace_kept=True)
        ms = time_steps(step, steps, 2, torch)
        fl = 4.0 * wl.Np * wl.topk * 64 * wl.d * wl.H * wl.B * (3.5 if backward else 1.0)
        out[name] = {"ms": round(ms, 4), "tflops": round(fl / (ms * 1e-3) / 1e12, 1),
                     "what": f"{'forward+backward' if backward else 'forward'}, B={wl.B} H={wl.H} Nc={wl.Nc} d={wl.d} "
                             f"topk={wl.topk}"}
        del buf, dev
        torch.cuda.empty_cache()

    run("mid_fwd_bwd", WORKLOADS["mid"], True, 20)
    w14 = WORKLOADS["wan14b"]
    run("wan14b_fwd", w14, False, 5)
    run("wan14b_fwd_bwd", w14, True, 3)
    run("wan14b_dense_fwd", Workload("wan14b_dense", w14.B, w14.H, w14.T, w14.Hh, w14.W, w14.d, w14.Nc), False, 2)
    out["wan14b_fwd_speedup_vs_dense"] = round(out["wan14b_dense_fwd"]["ms"] / out["wan14b_fwd"]["ms"], 2)
    # the pretraining sweep shape (B=2, 256 cubes), planted-locality inputs drawn on the host, at two
    # sparsities and both head dims, with the dense setting of the same shape as the reference
    for H, d in ((16, 128), (8, 64)):
        base = Workload(f"sweep_h{H}_d{d}", 2, H, 16, 32, 32, d, 32, planted=True)
        raw = synth.planted_inputs(base, 0)
        pb0 = vsa.problem_of(base)
        dev = {}
        for n, b in raw.items():
            src = torch.from_numpy(b.view("int16")).cuda().view(torch.bfloat16)
            dev[n] = torch.empty((base.B, base.H, base.Np, base.d), dtype=torch.bfloat16, device="cuda")
            vsa.vsa_tile_permute(pb0, src, dev[n])
        del raw
        a = (dev["q"], dev["k"], dev["v"], dev["gate_c"], dev["gate_f"])
        ms_by_k = {}
        for K in (32, 128, base.Nc):
            buf = vsa.Buffers(vsa.problem_of(base, topk=K))

            def step():
                buf.forward(*a)
                buf.backward(*a, dev["dout"], workspace_kept=True)
            ms_by_k[K] = time_steps(step, 10 if K < base.Nc else 3, 2, torch)
            del buf
        for K in (32, 128):
            fl = 3.5 * 4.0 * base.Np * K * 64 * d * H * 2
            out[f"sweep_h{H}_d{d}_k{K}_fwd_bwd"] = {
                "ms": round(ms_by_k[K], 4), "tflops": round(fl / (ms_by_k[K] * 1e-3) / 1e12, 1),
                "speedup_vs_dense": round(ms_by_k[base.Nc] / ms_by_k[K], 2), "ideal_speedup": base.Nc / K,
                "what": f"forward+backward, B=2 H={H} Nc=256 d={d} topk={K}, planted locality"}
        del dev
        torch.cuda.empty_cache()
    return out


def cpu_baseline(wl, seed):
    """The oracle (fp32 build, as it stands) on a few heads of the same workload, forward+backward."""
    # the only leg that touches the oracle (and the test helpers that wrap it)
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from oracle import vsa_oracle as orc
    from paper_2505_13389_amd.synth import Workload
    from helpers import grid_of, tiled_bits, widen
    heads = min(4, wl.H)  # about 10 s on the 16 host cores of the GPU machine
    one = Workload(wl.name + "_sample", 1, heads, wl.T, wl.Hh, wl.W, wl.d, wl.topk, wl.cube, wl.planted)
    x = widen(tiled_bits(one, seed))
    g = grid_of(one)
    t0 = time.perf_counter()
    f = orc.forward(g, x["q"], x["k"], x["v"], x["gate_c"], x["gate_f"], one.topk, real="f32")
    orc.backward(g, x["q"], x["k"], x["v"], x["gate_c"], x["gate_f"], x["dout"], f["block_idx"], one.topk, real="f32")
    sec = time.perf_counter() - t0
    flops = 3.5 * 4.0 * one.Np * one.topk * 64 * one.d * heads
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count()
    omp = os.environ.get("OMP_NUM_THREADS")
    if omp:
        cores = min(cores, int(omp))
    return {"value": flops / sec / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"{heads} of {wl.B * wl.H} (batch,head) slices of {wl.name}, forward+backward, fp32 oracle, "
                      f"{sec:.1f} s wall"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2505_13389_amd import vsa
    from paper_2505_13389_amd.synth import WORKLOADS, Workload
    problem_of = vsa.problem_of

    vsa.lib()  # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    wl = WORKLOADS[args.workload]
    if args.heads > 0:
        wl = Workload(f"{wl.name}_h{args.heads}", wl.B, args.heads, wl.T, wl.Hh, wl.W, wl.d, wl.topk, wl.cube, wl.planted)
    dev = device_inputs(wl, args.seed, torch)
    pb = problem_of(wl)
    buf = vsa.Buffers(pb)
    a = (dev["q"], dev["k"], dev["v"], dev["gate_c"], dev["gate_f"])

    def step():  # one layer's training step: the backward gets the workspace the forward left behind
        buf.forward(*a)
        buf.backward(*a, dev["dout"], workspace_kept=True)

    ms = time_steps(step, args.steps, args.warmup, torch)
    ms_fwd = time_steps(lambda: buf.forward(*a), args.steps, 1, torch)
    # the same step timed one by one (events), warm and with L2 / Infinity Cache swept before each
    per_step = sorted(event_times(step, args.steps, torch))
    sweep = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    cold = sorted(event_times(step, max(3, args.steps // 4), torch, before=lambda: sweep.fill_(1)))
    del sweep

    # the same steps again with every kernel bracketed by HIP events on the launch stream
    vsa.vsa_profile_begin(32 * args.steps)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    per = {}
    for name, t in vsa.vsa_profile_end():
        per.setdefault(name, []).append(t)
    kern = {n: sum(v) / len(v) * (len(v) / args.steps) for n, v in per.items()}  # ms per step, by kernel
    ms_profiled = sum(kern.values())

    fwd_flops = 4.0 * buf.Np * wl.topk * 64 * wl.d * wl.H * wl.B
    flops = 3.5 * fwd_flops
    tflops = flops / (ms * 1e-3) / 1e12
    pair_flops = 2.0 * 64 * 64 * wl.d
    pairs = wl.B * wl.H * buf.Nc * wl.topk
    dom = max(MATMULS, key=lambda n: kern.get(n, 0.0))
    launch_s = kern[dom] * 1e-3
    achieved = MATMULS[dom] * pair_flops * pairs / launch_s / 1e12
    executed = EXECUTED[dom] * pair_flops * pairs / launch_s / 1e12
    # compulsory bytes of that launch: each streamed and resident tensor once, outputs once
    tensor = wl.B * wl.H * buf.Np * wl.d * 2
    compulsory = {"fine_fwd": 7 * tensor, "fine_bwd_dq": 5 * tensor, "fine_bwd_dkv": 6 * tensor}[dom]
    gathered = pairs * 2 * 64 * wl.d * 2  # the two streamed 64 x d tiles of every pair, before any cache
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, TRAFFIC_FILE)
    if os.path.exists(tpath):
        tj = json.load(open(tpath))
        if tj.get("workload") == wl.name and dom in tj.get("kernels", {}):
            traffic = tj["kernels"][dom]["total_bytes"]
            traffic_source = (f"{TRAFFIC_FILE}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run "
                              f"({tj.get('measured_at', 'commit unknown')}), replayed here, not measured in this run")
    # The kernel is a dense bf16 contraction, so it is priced against the MFMA roof.  For the record:
    # the time this launch would take at each peak, on the matmuls it executes and on the bytes it
    # was measured to move across the L2 <-> fabric boundary (with i.i.d. selections the latter is
    # the longer one: the cache misses of the gather, not the algorithm's bytes).
    t_mfma = EXECUTED[dom] * pair_flops * pairs / (PEAK_BF16_TFLOPS * 1e12)
    t_hbm = (traffic if traffic is not None else compulsory) / (PEAK_HBM_GBS * 1e9)
    roofline = {"kernel": dom, "bound": "mfma", "achieved": round(achieved, 2),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                "traffic": traffic, "traffic_source": traffic_source,
                "achieved_executed_matmuls": round(executed, 2),
                "frac_executed_matmuls": round(executed / PEAK_BF16_TFLOPS, 4),
                "credited_matmuls_per_pair": MATMULS[dom], "executed_matmuls_per_pair": EXECUTED[dom],
                "algorithmic_bytes": compulsory, "gathered_bytes_before_cache": gathered,
                "traffic_over_algorithmic": None if traffic is None else round(traffic / compulsory, 2),
                "hbm_frac": None if traffic is None else round(traffic / launch_s / 1e9 / PEAK_HBM_GBS, 4),
                "ms_at_mfma_peak_on_executed_matmuls": round(t_mfma * 1e3, 4),
                "ms_at_hbm_peak_on_measured_traffic": round(t_hbm * 1e3, 4),
                "avg_launch_ms": round(kern[dom], 4)}

    # raster <-> tiled permutation of the 6 inputs and 6 outputs of a training step, timed apart
    def permutes():
        for n in ("q", "k", "v", "gate_c", "gate_f", "dout"):
            vsa.vsa_tile_permute(pb, dev["raster_" + n], dev[n], inverse=False)
        for t in (buf.out, buf.dq, buf.dk, buf.dv, buf.dgate_c, buf.dgate_f):
            vsa.vsa_tile_permute(pb, t, dev["raster_q"], inverse=True)
    raster_keep = dev["raster_q"].clone()
    ms_perm = time_steps(permutes, max(2, args.steps // 4), 1, torch)
    dev["raster_q"].copy_(raster_keep)

    rate = mfma_rate(torch, vsa)

    speedup = None
    if not args.no_dense:
        dense_wl = Workload(wl.name + "_dense", wl.B, wl.H, wl.T, wl.Hh, wl.W, wl.d, buf.Nc, wl.cube, wl.planted)
        dbuf = vsa.Buffers(problem_of(dense_wl))

        def dstep():
            dbuf.forward(*a)
            dbuf.backward(*a, dev["dout"], workspace_kept=True)
        ms_dense = time_steps(dstep, max(2, args.steps // 8), 1, torch)
        speedup = ms_dense / ms
        del dbuf

    line = {
        "metric": "VSA fwd+bwd effective TFLOP/s (selected blocks only)", "value": round(tflops, 2), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: B={wl.B} H={wl.H} grid={wl.T}x{wl.Hh}x{wl.W} (Np={buf.Np}, Nc={buf.Nc}) "
                               f"d={wl.d} topk={wl.topk}, forward+backward, tiled layout resident in HBM"},
        "pct_of_bf16_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2),
        "measured_mfma_tflops_random_operands": round(rate, 1),
        "pct_of_measured_mfma_rate": round(100.0 * tflops / rate, 2),
        "value_valid_tokens_only": round(tflops * (wl.L / buf.Np) ** 2, 2),
        "ms_per_step_median": round(per_step[len(per_step) // 2], 4), "ms_per_step_min": round(per_step[0], 4),
        "ms_per_step_cold_cache_median": round(cold[len(cold) // 2], 4),
        "fwd_ms": round(ms_fwd, 4), "fwd_tflops": round(fwd_flops / (ms_fwd * 1e-3) / 1e12, 2),
        "speedup_vs_dense": None if speedup is None else round(speedup, 2),
        "ideal_speedup_vs_dense": round(buf.Nc / wl.topk, 2),
        "permute_ms_12_tensors": round(ms_perm, 4),
        "ms_per_step_profiled": round(ms_profiled, 4),
        "kernel_ms": {n: round(t, 4) for n, t in sorted(kern.items(), key=lambda kv: -kv[1])},
        "roofline": roofline,
        # the HBM-bound steps: algorithmic bytes (every tensor once) / launch time, against 8 TB/s
        "hbm_bound_kernels": hbm_rates(wl, buf, kern, ms_perm),
    }
    if not args.no_configs:
        del buf, dev
        torch.cuda.empty_cache()
        line["configs"] = other_configs(torch, vsa, WORKLOADS, Workload, time_steps)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(wl, args.seed)
    print(json.dumps(line))


if __name__ == "__main__":
    main()

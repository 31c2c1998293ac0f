"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

Holds none of the attention arithmetic: only random draws, the bf16 rounding of the
inputs, and the named workload shapes.  Everything is produced in RASTER token order
[B,H,L,d] (L = T*Hh*W, n = t*Hh*W + h*W + w), as bf16 bit patterns (uint16), so that the
CPU oracle and the GPU library are handed identical bits.
"""
from dataclasses import dataclass

import numpy as np

BASE_SEED = 20250513


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    T: int
    Hh: int
    W: int
    d: int
    topk: int
    cube: tuple = (4, 4, 4)
    planted: bool = False

    @property
    def L(self):
        return self.T * self.Hh * self.W

    @property
    def padded(self):
        c = self.cube
        up = lambda a, b: (a + b - 1) // b * b
        return up(self.T, c[0]), up(self.Hh, c[1]), up(self.W, c[2])

    @property
    def Np(self):
        p = self.padded
        return p[0] * p[1] * p[2]

    @property
    def Nc(self):
        return self.Np // (self.cube[0] * self.cube[1] * self.cube[2])


# The named configurations (latent grids are the VALID grids; padding is the library's job).
WORKLOADS = {
    "tiny": Workload("tiny", 1, 2, 8, 16, 16, 64, 8),
    "tiny_dense": Workload("tiny_dense", 1, 2, 8, 16, 16, 64, 32),
    "mid": Workload("mid", 1, 12, 16, 32, 32, 128, 32),
    "wan1.3b": Workload("wan1.3b", 1, 12, 21, 30, 52, 128, 78),
    "wan14b": Workload("wan14b", 1, 40, 21, 45, 80, 128, 180),
    "sweep_h8_d64_k32": Workload("sweep_h8_d64_k32", 2, 8, 16, 32, 32, 64, 32, planted=True),
    "sweep_h16_d128_k32": Workload("sweep_h16_d128_k32", 2, 16, 16, 32, 32, 128, 32, planted=True),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even), returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def _rng(seed_offset: int):
    return np.random.Generator(np.random.PCG64(BASE_SEED + seed_offset))


def iid_inputs(wl: Workload, seed: int = 0, with_gate_f: bool = True):
    """Q,K,V,dO ~ N(0,1); gates ~ U(0,1).  Raster order, bf16 bits."""
    rng = _rng(seed)
    shape = (wl.B, wl.H, wl.L, wl.d)
    out = {}
    for name in ("q", "k", "v"):
        out[name] = f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))
    out["gate_c"] = f32_to_bf16_bits(rng.random(shape, dtype=np.float32))
    out["gate_f"] = f32_to_bf16_bits(rng.random(shape, dtype=np.float32)) if with_gate_f else None
    out["dout"] = f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))
    return out


def planted_inputs(wl: Workload, seed: int = 0, sigma: float = 0.5, gain: float = 3.0, sinks: int = 0,
                   with_gate_f: bool = True, sink_gain: float = 1.0):
    """Structured Q/K so that each query cube prefers its 3x3x3 neighbourhood of key cubes.

    Every cube gets a signature s_c ~ N(0,I).  Keys of cube c are s_c + sigma*eps; queries of
    cube c are gain * mean(s_c' over cubes within Chebyshev distance 1) + sigma*eps.  `sinks`
    cubes have `sink_gain` times their signature added to every query: every query cube then
    selects them, and (through the chance alignment of the other signatures with the sinks') the
    in-degrees of the remaining key cubes spread widely; the smaller sink_gain, the more the
    neighbourhood term shapes the rest of a list.
    """
    rng = _rng(1000 + seed)
    Ct, Ch, Cw = wl.cube
    Tp, Hp, Wp = wl.padded
    nt, nh, nw = Tp // Ct, Hp // Ch, Wp // Cw
    shape = (wl.B, wl.H, wl.L, wl.d)
    sig = rng.standard_normal((wl.B, wl.H, nt, nh, nw, wl.d), dtype=np.float32)
    # neighbourhood mean of signatures, clipped at the borders
    acc = np.zeros_like(sig)
    cnt = np.zeros((nt, nh, nw), dtype=np.float32)
    for dt in (-1, 0, 1):
        for dh in (-1, 0, 1):
            for dw in (-1, 0, 1):
                ts = slice(max(0, dt), nt + min(0, dt)); tt = slice(max(0, -dt), nt + min(0, -dt))
                hs = slice(max(0, dh), nh + min(0, dh)); ht = slice(max(0, -dh), nh + min(0, -dh))
                ws = slice(max(0, dw), nw + min(0, dw)); wt = slice(max(0, -dw), nw + min(0, -dw))
                acc[:, :, tt, ht, wt] += sig[:, :, ts, hs, ws]
                cnt[tt, ht, wt] += 1
    qsig = gain * acc / cnt[None, None, :, :, :, None]
    if sinks:
        flat = sig.reshape(wl.B, wl.H, -1, wl.d)
        pick = rng.choice(flat.shape[2], size=sinks, replace=False)
        qsig = qsig + sink_gain * flat[:, :, pick].sum(axis=2)[:, :, None, None, None, :]
    # cube coordinates of every raster token
    t, h, w = np.meshgrid(np.arange(wl.T), np.arange(wl.Hh), np.arange(wl.W), indexing="ij")
    ct, ch, cw = (t // Ct).ravel(), (h // Ch).ravel(), (w // Cw).ravel()
    k = sig[:, :, ct, ch, cw] + sigma * rng.standard_normal(shape, dtype=np.float32)
    q = qsig[:, :, ct, ch, cw] + sigma * rng.standard_normal(shape, dtype=np.float32)
    out = dict(q=f32_to_bf16_bits(q), k=f32_to_bf16_bits(k),
               v=f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32)),
               gate_c=f32_to_bf16_bits(rng.random(shape, dtype=np.float32)),
               gate_f=f32_to_bf16_bits(rng.random(shape, dtype=np.float32)) if with_gate_f else None,
               dout=f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32)))
    return out


def make_inputs(wl: Workload, seed: int = 0, with_gate_f: bool = True):
    if wl.planted:
        return planted_inputs(wl, seed, with_gate_f=with_gate_f)
    return iid_inputs(wl, seed, with_gate_f=with_gate_f)


def device_iid_inputs(wl: Workload, seed: int = 0, with_gate_f: bool = True, tiled_rows: int = None):
    """Same recipe as iid_inputs, drawn on the GPU with torch's seeded generator (for the large
    workloads, where drawing ~10^9 normals on the host would dominate a test).  Returns bf16
    tensors [B,H,rows,d] on the current device; rows = L (raster) unless `tiled_rows` is given
    (then the draw is directly in the padded tiled layout; pad rows hold ordinary draws, which
    the library must ignore)."""
    import torch
    g = torch.Generator(device="cuda")
    g.manual_seed(BASE_SEED + 5000 + seed)
    rows = wl.L if tiled_rows is None else tiled_rows
    shape = (wl.B, wl.H, rows, wl.d)
    out = {}
    for name in ("q", "k", "v", "dout"):
        out[name] = torch.randn(shape, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    out["gate_c"] = torch.rand(shape, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    out["gate_f"] = (torch.rand(shape, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
                     if with_gate_f else None)
    return out

"""ctypes binding of the plain CPU oracle for Video Sparse Attention (test infrastructure).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this module.
All arithmetic lives in vsa_oracle.c; this file only marshals numpy arrays.

Tensors are numpy arrays in TILED order, shape [B,H,Np,d]; `Grid` carries the geometry.
"""
import ctypes as C
from dataclasses import dataclass

import numpy as np

from . import build as _build

_LIBS = {}


def _lib(real: str):
    if real not in _LIBS:
        _build.build()
        lib = C.CDLL(_build.lib_path(real))
        lib.vsa_oracle_tiled_index.restype = C.c_int64
        lib.vsa_oracle_attention_flops.restype = C.c_double
        lib.vsa_oracle_attention_flops.argtypes = [C.c_double] * 5 + [C.c_int]
        _LIBS[real] = lib
    return _LIBS[real]


@dataclass(frozen=True)
class Grid:
    """Valid latent grid (T,Hh,W) and cube (Ct,Ch,Cw) [Sec. 2.2]."""
    T: int
    Hh: int
    W: int
    Ct: int = 4
    Ch: int = 4
    Cw: int = 4

    def args(self):
        return (self.T, self.Hh, self.W, self.Ct, self.Ch, self.Cw)

    @property
    def L(self):
        return self.T * self.Hh * self.W

    def dims(self):
        Np, Nc, Bk = C.c_int64(), C.c_int32(), C.c_int32()
        _lib("f64").vsa_oracle_dims(*self.args(), C.byref(Np), C.byref(Nc), C.byref(Bk))
        return Np.value, Nc.value, Bk.value

    @property
    def Np(self):
        return self.dims()[0]

    @property
    def Nc(self):
        return self.dims()[1]

    @property
    def Bk(self):
        return self.dims()[2]


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to float32 exactly."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


def _np_real(real):
    return np.float64 if real == "f64" else np.float32


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _as(a, dt):
    return None if a is None else np.ascontiguousarray(a, dtype=dt)


def tiled_index(grid: Grid, t: int, h: int, w: int) -> int:
    return int(_lib("f64").vsa_oracle_tiled_index(*grid.args(), t, h, w))


def valid_mask(grid: Grid):
    Np, Nc, _ = grid.dims()
    valid = np.zeros(Np, dtype=np.uint8)
    cnt = np.zeros(Nc, dtype=np.int32)
    _lib("f64").vsa_oracle_valid(*grid.args(), _ptr(valid), _ptr(cnt))
    return valid.astype(bool), cnt


def tile_u16(grid: Grid, src: np.ndarray, inverse: bool = False) -> np.ndarray:
    """Raster [B,H,L,d] -> tiled [B,H,Np,d] (or back) on 16-bit patterns; pads zero-filled."""
    assert src.dtype == np.uint16 and src.ndim == 4
    B, H, n, d = src.shape
    Np = grid.Np
    assert n == (Np if inverse else grid.L)
    src = np.ascontiguousarray(src)
    dst = np.empty((B, H, grid.L if inverse else Np, d), dtype=np.uint16)
    _lib("f64").vsa_oracle_tile_u16(*grid.args(), C.c_int64(B * H), d, _ptr(src), _ptr(dst), int(inverse))
    return dst


def forward(grid: Grid, q, k, v, gate_c, gate_f, topk: int, scale: float = None, block_idx=None,
            cubes=None, real: str = "f64", want_sc: bool = False):
    """Runs the oracle forward.  Returns a dict of numpy arrays.

    block_idx given -> used as the selection (indices-given mode).  cubes -> only those
    query cubes are evaluated (other rows of the outputs are left zero).
    """
    dt = _np_real(real)
    q, k, v, gate_c, gate_f = (_as(x, dt) for x in (q, k, v, gate_c, gate_f))
    B, H, Np, d = q.shape
    Np_, Nc, _ = grid.dims()
    assert Np == Np_
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    given = block_idx is not None
    idx = np.ascontiguousarray(block_idx, dtype=np.int32) if given else np.zeros((B, H, Nc, topk), np.int32)
    assert idx.shape == (B, H, Nc, topk)
    cub = None if cubes is None else np.ascontiguousarray(cubes, dtype=np.int32)
    res = dict(
        out=np.zeros((B, H, Np, d), dt), block_idx=idx, out_fine=np.zeros((B, H, Np, d), dt),
        lse_fine=np.zeros((B, H, Np), dt), out_coarse=np.zeros((B, H, Nc, d), dt),
        lse_coarse=np.zeros((B, H, Nc), dt), sc=np.zeros((B, H, Nc, Nc), dt) if want_sc else None)
    rc = _lib(real).vsa_oracle_forward(
        B, H, *grid.args(), d, topk, C.c_double(scale), int(given), _ptr(q), _ptr(k), _ptr(v), _ptr(gate_c),
        _ptr(gate_f), _ptr(cub), 0 if cub is None else len(cub), _ptr(res["out"]), _ptr(idx),
        _ptr(res["out_fine"]), _ptr(res["lse_fine"]), _ptr(res["out_coarse"]), _ptr(res["lse_coarse"]),
        _ptr(res["sc"]))
    if rc != 0:
        raise ValueError("vsa_oracle_forward: bad argument")
    return res


def backward(grid: Grid, q, k, v, gate_c, gate_f, dout, block_idx, topk: int, scale: float = None,
             real: str = "f64"):
    dt = _np_real(real)
    q, k, v, gate_c, gate_f, dout = (_as(x, dt) for x in (q, k, v, gate_c, gate_f, dout))
    B, H, Np, d = q.shape
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    idx = np.ascontiguousarray(block_idx, dtype=np.int32)
    res = dict(dq=np.zeros_like(q), dk=np.zeros_like(q), dv=np.zeros_like(q), dgate_c=np.zeros_like(q),
               dgate_f=None if gate_f is None else np.zeros_like(q))
    rc = _lib(real).vsa_oracle_backward(
        B, H, *grid.args(), d, topk, C.c_double(scale), _ptr(q), _ptr(k), _ptr(v), _ptr(gate_c), _ptr(gate_f),
        _ptr(dout), _ptr(idx), _ptr(res["dq"]), _ptr(res["dk"]), _ptr(res["dv"]), _ptr(res["dgate_c"]),
        _ptr(res["dgate_f"]))
    if rc != 0:
        raise ValueError("vsa_oracle_backward: bad argument")
    return res


def select_pooled(grid: Grid, q, k, topk: int, scale: float = None, real: str = "f64"):
    """Mismatched granularity [Sec. 3.2]: top-K of the coarse attention map average-pooled over (1,2,2)
    cubes.  Returns dict(tile_idx [B,H,Ns,topk], cube_idx [B,H,Nc,4*topk], pooled [B,H,Ns,Ns])."""
    dt = _np_real(real)
    q, k = _as(q, dt), _as(k, dt)
    B, H, Np, d = q.shape
    Np_, Nc, _ = grid.dims()
    assert Np == Np_
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    up = lambda a, b: (a + b - 1) // b
    Ns = up(grid.T, grid.Ct) * (up(grid.Hh, grid.Ch) // 2) * (up(grid.W, grid.Cw) // 2)
    res = dict(tile_idx=np.zeros((B, H, Ns, topk), np.int32), cube_idx=np.zeros((B, H, Nc, 4 * topk), np.int32),
               pooled=np.zeros((B, H, Ns, Ns), dt))
    rc = _lib(real).vsa_oracle_select_pooled(B, H, *grid.args(), d, topk, C.c_double(scale), _ptr(q), _ptr(k),
                                             _ptr(res["tile_idx"]), _ptr(res["cube_idx"]), _ptr(res["pooled"]))
    if rc != 0:
        raise ValueError("vsa_oracle_select_pooled: bad argument (odd number of cubes along h or w?)")
    return res


def block_mass(grid: Grid, q, k, scale: float = None, real: str = "f64"):
    """One (b,h) slice, q and k [Np,d] tiled: table [Nc,Nc] of the dense attention mass that the tokens
    of query cube c put on key cube j, averaged over the cube's valid tokens [Sec. 3.5]."""
    dt = _np_real(real)
    q, k = _as(q, dt), _as(k, dt)
    Np, d = q.shape
    Np_, Nc, _ = grid.dims()
    assert Np == Np_ and k.shape == q.shape
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    mass = np.zeros((Nc, Nc), dt)
    rc = _lib(real).vsa_oracle_block_mass(*grid.args(), d, C.c_double(scale), _ptr(q), _ptr(k), _ptr(mass))
    if rc != 0:
        raise ValueError("vsa_oracle_block_mass: bad argument")
    return mass


def keycubes(grid: Grid, kcube):
    """Key cubes (Kt,Kh,Kw) nested in the grid's cubes [Sec. 3.2, the 64 x 16 row of the tile-size
    tables]: (label [Np] of every tiled slot, -1 on pads; kcnt [Nk] valid tokens per key cube)."""
    Np, Nc, Bk = grid.dims()
    R = (grid.Ct // kcube[0]) * (grid.Ch // kcube[1]) * (grid.Cw // kcube[2])
    label = np.zeros(Np, np.int32)
    kcnt = np.zeros(Nc * R, np.int32)
    Nk = _lib("f64").vsa_oracle_keycubes(*grid.args(), *kcube, _ptr(label), _ptr(kcnt))
    if Nk != Nc * R:
        raise ValueError("vsa_oracle_keycubes: the key cube must divide the query cube")
    return label, kcnt


def forward_kq(grid: Grid, kcube, q, k, v, gate_c, gate_f, topk: int, scale: float = None, block_idx=None,
               cubes=None, real: str = "f64", want_sc: bool = False):
    """Forward with key cubes `kcube` = (Kt,Kh,Kw) smaller than the query cubes; block_idx [B,H,Nc,topk]
    names key cubes.  Otherwise as forward()."""
    dt = _np_real(real)
    q, k, v, gate_c, gate_f = (_as(x, dt) for x in (q, k, v, gate_c, gate_f))
    B, H, Np, d = q.shape
    Np_, Nc, _ = grid.dims()
    assert Np == Np_
    Nk = len(keycubes(grid, kcube)[1])
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    given = block_idx is not None
    idx = np.ascontiguousarray(block_idx, dtype=np.int32) if given else np.zeros((B, H, Nc, topk), np.int32)
    assert idx.shape == (B, H, Nc, topk)
    cub = None if cubes is None else np.ascontiguousarray(cubes, dtype=np.int32)
    res = dict(
        out=np.zeros((B, H, Np, d), dt), block_idx=idx, out_fine=np.zeros((B, H, Np, d), dt),
        lse_fine=np.zeros((B, H, Np), dt), out_coarse=np.zeros((B, H, Nc, d), dt),
        lse_coarse=np.zeros((B, H, Nc), dt), sc=np.zeros((B, H, Nc, Nk), dt) if want_sc else None)
    rc = _lib(real).vsa_oracle_forward_kq(
        B, H, *grid.args(), *kcube, d, topk, C.c_double(scale), int(given), _ptr(q), _ptr(k), _ptr(v), _ptr(gate_c),
        _ptr(gate_f), _ptr(cub), 0 if cub is None else len(cub), _ptr(res["out"]), _ptr(idx),
        _ptr(res["out_fine"]), _ptr(res["lse_fine"]), _ptr(res["out_coarse"]), _ptr(res["lse_coarse"]),
        _ptr(res["sc"]))
    if rc != 0:
        raise ValueError("vsa_oracle_forward_kq: bad argument")
    return res


def backward_kq(grid: Grid, kcube, q, k, v, gate_c, gate_f, dout, block_idx, topk: int, scale: float = None,
                real: str = "f64"):
    dt = _np_real(real)
    q, k, v, gate_c, gate_f, dout = (_as(x, dt) for x in (q, k, v, gate_c, gate_f, dout))
    B, H, Np, d = q.shape
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    idx = np.ascontiguousarray(block_idx, dtype=np.int32)
    res = dict(dq=np.zeros_like(q), dk=np.zeros_like(q), dv=np.zeros_like(q), dgate_c=np.zeros_like(q),
               dgate_f=None if gate_f is None else np.zeros_like(q))
    rc = _lib(real).vsa_oracle_backward_kq(
        B, H, *grid.args(), *kcube, d, topk, C.c_double(scale), _ptr(q), _ptr(k), _ptr(v), _ptr(gate_c),
        _ptr(gate_f), _ptr(dout), _ptr(idx), _ptr(res["dq"]), _ptr(res["dk"]), _ptr(res["dv"]),
        _ptr(res["dgate_c"]), _ptr(res["dgate_f"]))
    if rc != 0:
        raise ValueError("vsa_oracle_backward_kq: bad argument")
    return res


def attention_flops(n_query_tokens, n_key_tokens_per_query, d, heads, batch=1, with_backward=False) -> float:
    return float(_lib("f64").vsa_oracle_attention_flops(
        float(n_query_tokens), float(n_key_tokens_per_query), float(d), float(heads), float(batch),
        int(with_backward)))

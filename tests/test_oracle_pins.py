"""Pins of the CPU oracle against things other than itself (no GPU needed).

Each test names the fact that fixes the expected value: a closed form, brute force with a
numpy/torch library routine, an equivalence the paper states, or autograd / finite
differences for the backward.
"""
import os

import numpy as np
import pytest
import torch

from oracle import vsa_oracle as orc
from oracle.vsa_oracle import Grid

RNG = np.random.default_rng(7)


def rand(*shape):
    return RNG.standard_normal(shape)


def dense_attention(q, k, v, scale=None, key_valid=None):
    """Brute-force softmax attention in numpy fp64 [Sec. 2.1 attention equation, M = 0]."""
    d = q.shape[-1]
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    s = np.einsum("...id,...jd->...ij", q, k) * scale
    if key_valid is not None:
        s = np.where(key_valid, s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p /= p.sum(axis=-1, keepdims=True)
    return p @ v


def tile_np(grid, x):
    """Tile float arrays [B,H,L,d] -> [B,H,Np,d] by going through reshape/transpose (pads = 0).

    Independent second statement of the permutation: split each axis into (cube index,
    in-cube offset) and bring the three cube indices to the front [App. B tile()]."""
    B, H, L, d = x.shape
    Ct, Ch, Cw = grid.Ct, grid.Ch, grid.Cw
    Tp, Hp, Wp = -(-grid.T // Ct) * Ct, -(-grid.Hh // Ch) * Ch, -(-grid.W // Cw) * Cw
    full = np.zeros((B, H, Tp, Hp, Wp, d), x.dtype)
    full[:, :, :grid.T, :grid.Hh, :grid.W] = x.reshape(B, H, grid.T, grid.Hh, grid.W, d)
    y = full.reshape(B, H, Tp // Ct, Ct, Hp // Ch, Ch, Wp // Cw, Cw, d).transpose(0, 1, 2, 4, 6, 3, 5, 7, 8)
    return np.ascontiguousarray(y.reshape(B, H, Tp * Hp * Wp, d))


# ----------------------------------------------------------------------------- tile map
@pytest.mark.parametrize("grid", [Grid(8, 16, 16), Grid(4, 8, 12, 2, 2, 2), Grid(5, 6, 7, 4, 4, 4),
                                  Grid(3, 5, 2, 1, 1, 1), Grid(21, 30, 52)])
def test_tile_map_is_a_bijection_and_matches_reshape_transpose(grid):
    Np, Nc, Bk = grid.dims()
    idx = np.array([orc.tiled_index(grid, t, h, w) for t in range(grid.T) for h in range(grid.Hh)
                    for w in range(grid.W)], dtype=np.int64)
    assert len(np.unique(idx)) == grid.L and idx.min() >= 0 and idx.max() < Np
    # reshape/transpose statement of the same permutation
    marks = np.arange(1, grid.L + 1, dtype=np.float64).reshape(1, 1, grid.L, 1)
    tiled = tile_np(grid, marks)[0, 0, :, 0]
    assert np.array_equal(tiled[idx], np.arange(1, grid.L + 1))
    valid, cnt = orc.valid_mask(grid)
    assert np.array_equal(valid, tiled != 0)
    assert np.array_equal(cnt, (tiled != 0).reshape(Nc, Bk).sum(axis=1))
    assert cnt.min() >= 1  # padding to the next cube multiple never leaves an empty cube


def test_tile_map_identity_for_unit_cube():
    grid = Grid(3, 4, 5, 1, 1, 1)
    idx = [orc.tiled_index(grid, t, h, w) for t in range(3) for h in range(4) for w in range(5)]
    assert idx == list(range(60))


@pytest.mark.parametrize("grid", [Grid(8, 16, 16), Grid(5, 6, 7), Grid(4, 4, 6, 2, 2, 2)])
def test_tile_untile_round_trip_bit_exact(grid):
    src = RNG.integers(0, 65536, size=(2, 3, grid.L, 8), dtype=np.uint16)
    tiled = orc.tile_u16(grid, src)
    assert tiled.shape == (2, 3, grid.Np, 8)
    back = orc.tile_u16(grid, tiled, inverse=True)
    assert np.array_equal(back, src)
    valid, _ = orc.valid_mask(grid)
    assert not tiled[:, :, ~valid].any()
    ref = tile_np(grid, src.astype(np.float64))
    assert np.array_equal(tiled.astype(np.float64), ref)


# ----------------------------------------------------------------------------- pooling + coarse
def test_unit_cube_coarse_stage_is_dense_attention():
    """Cube (1,1,1): pooling is the identity, so O_c is plain dense attention [Sec. 2.1]."""
    grid = Grid(2, 3, 4, 1, 1, 1)
    q, k, v = rand(2, 2, 24, 8), rand(2, 2, 24, 8), rand(2, 2, 24, 8)
    g = rand(2, 2, 24, 8)
    r = orc.forward(grid, q, k, v, g, g, topk=5, want_sc=True)
    ref = dense_attention(q, k, v)
    assert np.abs(r["out_coarse"] - ref).max() < 1e-12
    s = np.einsum("bhid,bhjd->bhij", q, k) / np.sqrt(8)
    assert np.abs(r["sc"] - s).max() < 1e-12
    lse = np.log(np.exp(s).sum(-1))
    assert np.abs(r["lse_coarse"] - lse).max() < 1e-12


def test_pooling_mean_closed_forms():
    grid = Grid(4, 4, 8)  # two cubes
    Np, Nc, Bk = grid.dims()
    d = 4
    # constant per cube -> pooled value is that constant; A_c V_c then mixes the two constants
    v = np.zeros((1, 1, Np, d)); v[0, 0, :64] = 3.0; v[0, 0, 64:] = -1.0
    # q = k = arange pattern: the mean of an arithmetic progression is its midpoint
    x = np.zeros((1, 1, Np, d))
    x[0, 0, :64, :] = np.arange(64)[:, None]          # mean 31.5
    x[0, 0, 64:, :] = 2.0 * np.arange(64)[:, None]    # mean 63
    g = np.ones((1, 1, Np, d))
    r = orc.forward(grid, x, x, v, g, g, topk=2, scale=0.001, want_sc=True)
    sc = np.array([[31.5 * 31.5, 31.5 * 63], [63 * 31.5, 63 * 63]]) * d * 0.001
    assert np.abs(r["sc"][0, 0] - sc).max() < 1e-9
    a = np.exp(sc - sc.max(1, keepdims=True)); a /= a.sum(1, keepdims=True)
    oc = a @ np.array([[3.0] * d, [-1.0] * d])
    assert np.abs(r["out_coarse"][0, 0] - oc).max() < 1e-12


def test_coarse_rows_sum_to_one():
    grid = Grid(8, 8, 8)
    Np = grid.Np
    q, k, v = rand(1, 2, Np, 16), rand(1, 2, Np, 16), rand(1, 2, Np, 16)
    r = orc.forward(grid, q, k, v, q, q, topk=3, want_sc=True)
    assert np.abs(np.exp(r["sc"] - r["lse_coarse"][..., None]).sum(-1) - 1).max() < 1e-12


# ----------------------------------------------------------------------------- top-K
def brute_topk(sc, K):
    order = np.argsort(-sc, axis=-1, kind="stable")  # stable: equal values keep index order
    return np.sort(order[..., :K], axis=-1)


@pytest.mark.parametrize("real", ["f64", "f32"])
def test_topk_matches_full_sort(real):
    grid = Grid(8, 16, 16)
    Np, Nc, _ = grid.dims()
    q, k, v = rand(1, 2, Np, 16), rand(1, 2, Np, 16), rand(1, 2, Np, 16)
    for K in (1, 5, 31, 32):
        r = orc.forward(grid, q, k, v, q, q, topk=K, want_sc=True, real=real)
        assert np.array_equal(r["block_idx"], brute_topk(r["sc"], K))
        assert (np.diff(r["block_idx"], axis=-1) > 0).all()
    assert np.array_equal(r["block_idx"][0, 0, 0], np.arange(Nc))  # K = Nc: every cube


def test_topk_ties_go_to_lower_index():
    grid = Grid(8, 8, 8)
    Np = grid.Np
    z = np.zeros((1, 1, Np, 8))
    r = orc.forward(grid, z, rand(1, 1, Np, 8), rand(1, 1, Np, 8), z, z, topk=3)
    assert np.array_equal(r["block_idx"][0, 0], np.tile(np.arange(3), (8, 1)))


# ----------------------------------------------------------------------------- fine + combine
@pytest.mark.parametrize("real,tol", [("f64", 1e-12), ("f32", 2e-5)])
def test_all_tiles_selected_equals_dense_attention(real, tol):
    """K = number of tiles, G_c = 0, G_f = 1: VSA is full attention [Sec. 2.3]."""
    grid = Grid(4, 8, 8)
    Np, Nc, _ = grid.dims()
    q, k, v = rand(1, 2, Np, 16), rand(1, 2, Np, 16), rand(1, 2, Np, 16)
    zero, one = np.zeros_like(q), np.ones_like(q)
    r = orc.forward(grid, q, k, v, zero, one, topk=Nc, real=real)
    ref = dense_attention(q, k, v)
    assert np.abs(r["out"] - ref).max() < tol
    assert np.abs(r["out_fine"] - ref).max() < tol
    s = np.einsum("bhid,bhjd->bhij", q, k) / 4.0
    assert np.abs(r["lse_fine"] - np.log(np.exp(s).sum(-1))).max() < tol * 10
    # gate_f = NULL means ones
    r2 = orc.forward(grid, q, k, v, zero, None, topk=Nc, real=real)
    assert np.array_equal(r2["out"], r["out"])


def test_unit_cube_small_k_is_attention_over_the_topk_keys():
    grid = Grid(2, 3, 5, 1, 1, 1)
    L, d, K = 30, 8, 4
    q, k, v = rand(1, 1, L, d), rand(1, 1, L, d), rand(1, 1, L, d)
    gc, gf = rand(1, 1, L, d), rand(1, 1, L, d)
    r = orc.forward(grid, q, k, v, gc, gf, topk=K)
    s = (q[0, 0] @ k[0, 0].T) / np.sqrt(d)
    ref_f = np.zeros((L, d))
    for i in range(L):
        keep = np.argsort(-s[i], kind="stable")[:K]
        p = np.exp(s[i, keep] - s[i, keep].max()); p /= p.sum()
        ref_f[i] = p @ v[0, 0, keep]
    assert np.abs(r["out_fine"][0, 0] - ref_f).max() < 1e-12
    full = dense_attention(q, k, v)[0, 0]
    assert np.abs(r["out"][0, 0] - (full * gc[0, 0] + ref_f * gf[0, 0])).max() < 1e-12
    # K = L: O = (G_c + G_f) * Attn(Q,K,V)
    r = orc.forward(grid, q, k, v, gc, gf, topk=L)
    assert np.abs(r["out"][0, 0] - (gc[0, 0] + gf[0, 0]) * full).max() < 1e-12


def test_constant_values_pass_through():
    grid = Grid(8, 8, 8)
    Np = grid.Np
    q, k = rand(1, 1, Np, 8), rand(1, 1, Np, 8)
    v0 = rand(8)
    v = np.broadcast_to(v0, (1, 1, Np, 8)).copy()
    gc, gf = rand(1, 1, Np, 8), rand(1, 1, Np, 8)
    r = orc.forward(grid, q, k, v, gc, gf, topk=3)
    assert np.abs(r["out_fine"] - v0).max() < 1e-12
    assert np.abs(r["out"] - (gc + gf) * v0).max() < 1e-12


def test_given_indices_are_used_verbatim():
    grid = Grid(4, 8, 8)
    Np, Nc, Bk = grid.dims()
    q, k, v = rand(1, 1, Np, 8), rand(1, 1, Np, 8), rand(1, 1, Np, 8)
    idx = np.sort(np.stack([RNG.choice(Nc, 2, replace=False) for _ in range(Nc)]), axis=-1).reshape(1, 1, Nc, 2)
    one = np.ones_like(q)
    r = orc.forward(grid, q, k, v, 0 * one, one, topk=2, block_idx=idx.astype(np.int32))
    for c in range(Nc):
        keys = np.concatenate([np.arange(j * Bk, (j + 1) * Bk) for j in idx[0, 0, c]])
        ref = dense_attention(q[0, 0, c * Bk:(c + 1) * Bk], k[0, 0, keys], v[0, 0, keys])
        assert np.abs(r["out"][0, 0, c * Bk:(c + 1) * Bk] - ref).max() < 1e-12


# ----------------------------------------------------------------------------- pads
def test_padded_grid_all_tiles_equals_dense_attention_over_valid_tokens():
    grid = Grid(5, 6, 7)  # pads in every axis
    Np, Nc, _ = grid.dims()
    d = 8
    qr, kr, vr = rand(1, 2, grid.L, d), rand(1, 2, grid.L, d), rand(1, 2, grid.L, d)
    q, k, v = tile_np(grid, qr), tile_np(grid, kr), tile_np(grid, vr)
    valid, _ = orc.valid_mask(grid)
    one = np.ones_like(q)
    r = orc.forward(grid, q, k, v, 0 * one, one, topk=Nc)
    ref = tile_np(grid, dense_attention(qr, kr, vr))
    assert np.abs(r["out"] - ref).max() < 1e-12
    assert not r["out"][:, :, ~valid].any()
    # garbage in the pad slots changes nothing, forward or backward
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    for a in (q2, k2, v2):
        a[:, :, ~valid] = 1e3 * rand(*a[:, :, ~valid].shape)
    gc, gf, do = rand(*q.shape), rand(*q.shape), rand(*q.shape)
    ra = orc.forward(grid, q, k, v, gc, gf, topk=3)
    rb = orc.forward(grid, q2, k2, v2, gc, gf, topk=3)
    assert np.array_equal(ra["block_idx"], rb["block_idx"]) and np.array_equal(ra["out"], rb["out"])
    do2 = do.copy(); do2[:, :, ~valid] = 77.0
    ba = orc.backward(grid, q, k, v, gc, gf, do, ra["block_idx"], 3)
    bb = orc.backward(grid, q2, k2, v2, gc, gf, do2, ra["block_idx"], 3)
    for name in ba:
        assert np.array_equal(ba[name], bb[name]), name
        assert not ba[name][:, :, ~valid].any(), name


# ----------------------------------------------------------------------------- backward
def torch_vsa(grid, q, k, v, gc, gf, idx, scale):
    """Independent forward in torch fp64 (tiled layout, indices frozen), for autograd.

    Written from the method description [Sec. 2.2]: masked mean pooling, cube-level softmax
    attention broadcast back to tokens, token-level softmax under the block mask built from
    the index list, gated sum."""
    Np, Nc, Bk = grid.dims()
    valid_np, cnt_np = orc.valid_mask(grid)
    valid = torch.from_numpy(valid_np)
    cnt = torch.from_numpy(cnt_np).double()
    B, H, _, d = q.shape
    vm = valid.view(1, 1, Nc, Bk, 1).double()
    pool = lambda x: (x.view(B, H, Nc, Bk, d) * vm).sum(3) / cnt.view(1, 1, Nc, 1)
    qc, kc, vc = pool(q), pool(k), pool(v)
    ac = torch.softmax(qc @ kc.transpose(-1, -2) * scale, dim=-1)
    oc = (ac @ vc).repeat_interleave(Bk, dim=2)
    block = torch.zeros(B, H, Nc, Nc, dtype=torch.bool)
    block.scatter_(-1, torch.from_numpy(idx).long(), True)
    mask = block.repeat_interleave(Bk, 2).repeat_interleave(Bk, 3) & valid.view(1, 1, 1, Np)
    s = (q @ k.transpose(-1, -2) * scale).masked_fill(~mask, float("-inf"))
    of = torch.softmax(s, dim=-1) @ v
    out = oc * gc + of * (gf if gf is not None else 1.0)
    return out * valid.view(1, 1, Np, 1)


@pytest.mark.parametrize("grid,topk,with_gf", [(Grid(4, 8, 8), 2, True), (Grid(4, 8, 8), 4, False),
                                               (Grid(5, 6, 7), 3, True), (Grid(2, 4, 6, 2, 2, 2), 2, True)])
def test_backward_matches_torch_autograd(grid, topk, with_gf):
    Np, Nc, Bk = grid.dims()
    B, H, d = 1, 2, 8
    valid, _ = orc.valid_mask(grid)
    arrs = [rand(B, H, Np, d) * valid[None, None, :, None] for _ in range(6)]
    q, k, v, gc, gf, do = arrs
    if not with_gf:
        gf = None
    scale = 0.3
    f = orc.forward(grid, q, k, v, gc, gf, topk, scale=scale)
    idx = f["block_idx"]
    tq, tk, tv, tgc = (torch.from_numpy(x).requires_grad_(True) for x in (q, k, v, gc))
    tgf = torch.from_numpy(gf).requires_grad_(True) if with_gf else None
    out = torch_vsa(grid, tq, tk, tv, tgc, tgf, idx, scale)
    assert np.abs(out.detach().numpy() - f["out"]).max() < 1e-12
    (out * torch.from_numpy(do)).sum().backward()
    b = orc.backward(grid, q, k, v, gc, gf, do, idx, topk, scale=scale)
    vm = valid[None, None, :, None]
    assert np.abs(b["dq"] - tq.grad.numpy() * vm).max() < 1e-11
    assert np.abs(b["dk"] - tk.grad.numpy() * vm).max() < 1e-11
    assert np.abs(b["dv"] - tv.grad.numpy() * vm).max() < 1e-11
    assert np.abs(b["dgate_c"] - tgc.grad.numpy()).max() < 1e-11
    if with_gf:
        assert np.abs(b["dgate_f"] - tgf.grad.numpy()).max() < 1e-11
    else:
        assert b["dgate_f"] is None


def test_backward_matches_central_finite_differences():
    grid = Grid(4, 4, 8)
    Np, Nc, Bk = grid.dims()
    B, H, d, topk = 1, 1, 4, 1
    q, k, v, gc, gf, do = (rand(B, H, Np, d) for _ in range(6))
    f = orc.forward(grid, q, k, v, gc, gf, topk)
    idx = f["block_idx"]
    b = orc.backward(grid, q, k, v, gc, gf, do, idx, topk)
    names = ["q", "k", "v", "gate_c", "gate_f"]
    tens = dict(q=q, k=k, v=v, gate_c=gc, gate_f=gf)
    loss = lambda t: float((orc.forward(grid, t["q"], t["k"], t["v"], t["gate_c"], t["gate_f"], topk,
                                        block_idx=idx)["out"] * do).sum())
    h = 1e-5
    for name in names:
        for _ in range(6):
            pos = tuple(RNG.integers(0, s) for s in tens[name].shape)
            save = tens[name][pos]
            tens[name][pos] = save + h; lp = loss(tens)
            tens[name][pos] = save - h; lm = loss(tens)
            tens[name][pos] = save
            fd = (lp - lm) / (2 * h)
            assert abs(fd - b["d" + name][pos]) < 1e-6 * max(1.0, abs(fd)), (name, pos)


def test_dense_selection_gradients_equal_dense_attention_gradients():
    """K = all tiles, G_c = 0, G_f absent: gradients of plain softmax attention (torch autograd)."""
    grid = Grid(4, 4, 8)
    Np, Nc, _ = grid.dims()
    q, k, v, do = (rand(1, 2, Np, 8) for _ in range(4))
    f = orc.forward(grid, q, k, v, 0 * q, None, Nc)
    b = orc.backward(grid, q, k, v, 0 * q, None, do, f["block_idx"], Nc)
    tq, tk, tv = (torch.from_numpy(x).requires_grad_(True) for x in (q, k, v))
    o = torch.softmax(tq @ tk.transpose(-1, -2) / np.sqrt(8), -1) @ tv
    (o * torch.from_numpy(do)).sum().backward()
    for name, t in (("dq", tq), ("dk", tk), ("dv", tv)):
        assert np.abs(b[name] - t.grad.numpy()).max() < 1e-12, name


# ----------------------------------------------------------------------------- fp32 build, anchors
def test_fp32_build_stays_close_to_fp64_build():
    grid = Grid(8, 8, 8)
    Np = grid.Np
    q, k, v, gc, gf, do = (rand(1, 2, Np, 16).astype(np.float32) for _ in range(6))
    a = orc.forward(grid, q, k, v, gc, gf, 3, real="f64")
    b = orc.forward(grid, q, k, v, gc, gf, 3, block_idx=a["block_idx"], real="f32")
    assert np.abs(a["out"] - b["out"]).max() < 1e-5
    ga = orc.backward(grid, q, k, v, gc, gf, do, a["block_idx"], 3, real="f64")
    gb = orc.backward(grid, q, k, v, gc, gf, do, a["block_idx"], 3, real="f32")
    for name in ga:
        assert np.abs(ga[name] - gb[name]).max() < 2e-5, name


# ----------------------------------------------------------------------------- selection quality
def test_block_mass_is_the_dense_attention_matrix_summed_over_cubes():
    """[Sec. 3.5] the mass table is the dense attention matrix (numpy brute force over the valid keys)
    summed over key cubes and averaged over the valid tokens of each query cube: rows sum to 1; for
    the unit cube it IS the attention matrix; q = 0 gives each key cube its share of the valid tokens."""
    g = Grid(5, 6, 7, 4, 4, 4)  # ragged on every axis
    valid, cnt = orc.valid_mask(g)
    Np, Nc, Bk = g.dims()
    d = 16
    q, k = rand(Np, d), rand(Np, d)
    mass = orc.block_mass(g, q, k)
    s = (q @ k.T) / np.sqrt(d)
    s = np.where(valid[None, :], s, -np.inf)
    p = np.exp(s - s.max(-1, keepdims=True))
    p /= p.sum(-1, keepdims=True)
    p = p * valid[:, None]
    want = p.reshape(Nc, Bk, Nc, Bk).sum(axis=(1, 3)) / cnt[:, None]
    assert np.abs(mass - want).max() < 1e-12
    assert np.abs(mass.sum(-1) - 1.0).max() < 1e-12
    uniform = orc.block_mass(g, np.zeros_like(q), k)
    assert np.abs(uniform - (cnt / cnt.sum())[None, :]).max() < 1e-12
    g1 = Grid(2, 3, 4, 1, 1, 1)
    q1, k1 = rand(24, 8), rand(24, 8)
    s1 = (q1 @ k1.T) / np.sqrt(8)
    p1 = np.exp(s1 - s1.max(-1, keepdims=True))
    assert np.abs(orc.block_mass(g1, q1, k1) - p1 / p1.sum(-1, keepdims=True)).max() < 1e-12


# ----------------------------------------------------------------------------- mismatched granularity
def test_pooled_selection_is_topk_of_the_block_averaged_attention_map():
    """[Sec. 3.2] numpy restatement: softmax of the pooled logits, mean over the 2x2 groups of cubes on
    both axes by reshape, stable argsort; the expanded cube lists hold exactly the four cubes of each
    selected tile.  With q = 0 the map is flat and the first K tiles win (ties to the lower index)."""
    g = Grid(8, 14, 15, 4, 4, 4)  # 2 x 4 x 4 cubes, ragged in h and w
    valid, cnt = orc.valid_mask(g)
    Np, Nc, Bk = g.dims()
    d, K = 16, 3
    Nt, Nh, Nw = 2, 4, 4
    q, k = rand(1, 2, Np, d), rand(1, 2, Np, d)
    got = orc.select_pooled(g, q, k, K)
    for h in range(2):
        pool = lambda x: (x[0, h] * valid[:, None]).reshape(Nc, Bk, d).sum(1) / cnt[:, None]
        s = pool(q) @ pool(k).T / np.sqrt(d)
        p = np.exp(s - s.max(-1, keepdims=True))
        p /= p.sum(-1, keepdims=True)
        ps = p.reshape(Nt, Nh // 2, 2, Nw // 2, 2, Nt, Nh // 2, 2, Nw // 2, 2).mean(axis=(2, 4, 7, 9)).reshape(8, 8)
        assert np.abs(got["pooled"][0, h] - ps).max() < 1e-14
        want = np.sort(np.argsort(-ps, axis=-1, kind="stable")[:, :K], axis=-1)
        assert np.array_equal(got["tile_idx"][0, h], want)
        for c in range(Nc):
            ct, ch, cw = c // (Nh * Nw), (c // Nw) % Nh, c % Nw
            sq = (ct * (Nh // 2) + ch // 2) * (Nw // 2) + cw // 2
            cubes = set()
            for s_ in want[sq]:
                st, sh, sw = s_ // 4, (s_ // 2) % 2, s_ % 2
                cubes |= {(st * Nh + 2 * sh + a) * Nw + 2 * sw + b for a in (0, 1) for b in (0, 1)}
            assert set(got["cube_idx"][0, h, c]) == cubes and len(cubes) == 4 * K
            assert (np.diff(got["cube_idx"][0, h, c]) > 0).all()
    flat = orc.select_pooled(g, np.zeros_like(q), k, K)
    assert np.array_equal(flat["tile_idx"], np.broadcast_to(np.arange(K, dtype=np.int32), flat["tile_idx"].shape))
    with pytest.raises(ValueError):
        orc.select_pooled(Grid(8, 12, 16, 4, 4, 4), rand(1, 1, 1536, 8), rand(1, 1, 1536, 8), 2)  # 3 cubes along h


# ----------------------------------------------------------------------------- key cubes smaller than query cubes
def keycube_labels_np(grid, kcube):
    """The key-cube label of every tiled slot by reshape/transpose: number the key cubes on the padded
    grid (query cube major, then the key cube inside it), broadcast over their tokens, tile."""
    Ct, Ch, Cw = grid.Ct, grid.Ch, grid.Cw
    Kt, Kh, Kw = kcube
    Tp, Hp, Wp = -(-grid.T // Ct) * Ct, -(-grid.Hh // Ch) * Ch, -(-grid.W // Cw) * Cw
    nt, nh, nw, rt, rh, rw = Tp // Ct, Hp // Ch, Wp // Cw, Ct // Kt, Ch // Kh, Cw // Kw
    ids = np.arange(nt * nh * nw * rt * rh * rw).reshape(nt, nh, nw, rt, rh, rw)   # [cube..., local...]
    full = ids.transpose(0, 3, 1, 4, 2, 5)                                        # (nt, rt, nh, rh, nw, rw)
    full = np.repeat(np.repeat(np.repeat(full, Kt, 1), Kh, 3), Kw, 5).reshape(Tp, Hp, Wp)
    lab = np.full((Tp, Hp, Wp), -1)
    lab[:grid.T, :grid.Hh, :grid.W] = full[:grid.T, :grid.Hh, :grid.W]
    y = lab.reshape(nt, Ct, nh, Ch, nw, Cw).transpose(0, 2, 4, 1, 3, 5)
    return y.reshape(-1)


@pytest.mark.parametrize("grid,kcube", [(Grid(8, 8, 8), (2, 4, 2)), (Grid(5, 6, 7), (2, 4, 2)),
                                        (Grid(4, 8, 6, 2, 4, 2), (1, 2, 2)), (Grid(4, 4, 8), (4, 4, 4))])
def test_key_cube_labels_match_reshape_transpose(grid, kcube):
    label, kcnt = orc.keycubes(grid, kcube)
    want = keycube_labels_np(grid, kcube)
    assert np.array_equal(label, want)
    assert np.array_equal(kcnt, np.bincount(want[want >= 0], minlength=len(kcnt)))
    valid, _ = orc.valid_mask(grid)
    assert np.array_equal(label >= 0, valid)


def test_key_cubes_equal_to_query_cubes_give_the_ordinary_method():
    grid = Grid(5, 6, 7)
    Np, Nc, Bk = grid.dims()
    B, H, d, topk = 1, 2, 8, 3
    valid, _ = orc.valid_mask(grid)
    q, k, v, gc, gf, do = [rand(B, H, Np, d) * valid[None, None, :, None] for _ in range(6)]
    a = orc.forward(grid, q, k, v, gc, gf, topk, want_sc=True)
    b = orc.forward_kq(grid, (4, 4, 4), q, k, v, gc, gf, topk, want_sc=True)
    assert np.array_equal(a["block_idx"], b["block_idx"])
    for name in ("out", "out_fine", "lse_fine", "out_coarse", "lse_coarse", "sc"):
        assert np.abs(a[name] - b[name]).max() < 1e-12, name
    ga = orc.backward(grid, q, k, v, gc, gf, do, a["block_idx"], topk)
    gb = orc.backward_kq(grid, (4, 4, 4), q, k, v, gc, gf, do, a["block_idx"], topk)
    for name in ga:
        assert np.abs(ga[name] - gb[name]).max() < 1e-12, name


def test_key_cubes_all_selected_equals_dense_attention_over_valid_tokens():
    grid, kcube = Grid(5, 6, 7), (2, 4, 2)   # the padded grid holds dead key cubes (t = 6, 7 are all pad)
    Np, Nc, Bk = grid.dims()
    label, kcnt = orc.keycubes(grid, kcube)
    live = int((kcnt > 0).sum())
    assert live < len(kcnt)
    valid, _ = orc.valid_mask(grid)
    B, H, d = 1, 2, 8
    q, k, v = [rand(B, H, Np, d) * valid[None, None, :, None] for _ in range(3)]
    ones = np.ones_like(q)
    f = orc.forward_kq(grid, kcube, q, k, v, np.zeros_like(q), ones, live, want_sc=True)
    assert np.array_equal(f["block_idx"][0, 0, 0], np.flatnonzero(kcnt > 0))
    want = dense_attention(q, k, v, key_valid=valid[None, None, None, :]) * valid[None, None, :, None]
    assert np.abs(f["out"] - want).max() < 1e-12
    assert np.isneginf(f["sc"][..., kcnt == 0]).all() and np.isfinite(f["sc"][..., kcnt > 0]).all()
    with pytest.raises(ValueError):
        orc.forward_kq(grid, kcube, q, k, v, ones, ones, live + 1)


def test_key_cube_lists_that_name_whole_cubes_give_the_fine_stage_of_the_ordinary_method():
    grid, kcube = Grid(4, 8, 8), (2, 4, 2)
    Np, Nc, Bk = grid.dims()
    B, H, d, topk = 1, 2, 8, 2
    q, k, v, gc, gf, do = [rand(B, H, Np, d) for _ in range(6)]
    a = orc.forward(grid, q, k, v, gc, gf, topk)
    sub = (a["block_idx"][..., None] * 4 + np.arange(4)).reshape(B, H, Nc, 4 * topk)
    b = orc.forward_kq(grid, kcube, q, k, v, gc, gf, 4 * topk, block_idx=sub)
    assert np.abs(a["out_fine"] - b["out_fine"]).max() < 1e-12 and np.abs(a["lse_fine"] - b["lse_fine"]).max() < 1e-12


def torch_vsa_kq(grid, kcube, q, k, v, gc, gf, idx, scale):
    """torch fp64 restatement with key cubes [Sec. 2.2 with the key side pooled and selected in smaller
    cubes]: membership matrices instead of loops, indices frozen."""
    Np, Nc, Bk = grid.dims()
    label_np = keycube_labels_np(grid, kcube)
    Nk = Nc * (grid.Ct // kcube[0]) * (grid.Ch // kcube[1]) * (grid.Cw // kcube[2])
    label = torch.from_numpy(label_np)
    valid = label >= 0
    B, H, _, d = q.shape
    memb_k = (label.view(1, Np) == torch.arange(Nk).view(Nk, 1)).double()         # [Nk, Np]
    memb_q = ((torch.arange(Np) // Bk).view(1, Np) == torch.arange(Nc).view(Nc, 1)).double() * valid.double()
    kcnt = memb_k.sum(1)
    qc = memb_q @ q / memb_q.sum(1).view(Nc, 1)
    kc = memb_k @ k / kcnt.clamp(min=1).view(Nk, 1)
    vc = memb_k @ v / kcnt.clamp(min=1).view(Nk, 1)
    sc = (qc @ kc.transpose(-1, -2) * scale).masked_fill(kcnt.view(1, 1, 1, Nk) == 0, float("-inf"))
    oc = (torch.softmax(sc, dim=-1) @ vc).repeat_interleave(Bk, dim=2)
    block = torch.zeros(B, H, Nc, Nk, dtype=torch.bool)
    block.scatter_(-1, torch.from_numpy(idx).long(), True)
    lab = label.clamp(min=0)
    mask = block.repeat_interleave(Bk, 2)[..., lab] & valid.view(1, 1, 1, Np)
    s = (q @ k.transpose(-1, -2) * scale).masked_fill(~mask, float("-inf"))
    of = torch.softmax(s, dim=-1) @ v
    out = oc * gc + of * (gf if gf is not None else 1.0)
    return out * valid.view(1, 1, Np, 1)


@pytest.mark.parametrize("grid,kcube,topk,with_gf", [(Grid(4, 8, 8), (2, 4, 2), 5, True), (Grid(5, 6, 7), (2, 4, 2), 7, True),
                                                     (Grid(5, 6, 7), (2, 4, 2), 3, False), (Grid(4, 4, 6, 2, 2, 2), (1, 2, 1), 6, True)])
def test_key_cube_forward_and_backward_match_torch_autograd(grid, kcube, topk, with_gf):
    Np, Nc, Bk = grid.dims()
    B, H, d = 1, 2, 8
    valid, _ = orc.valid_mask(grid)
    q, k, v, gc, gf, do = [rand(B, H, Np, d) * valid[None, None, :, None] for _ in range(6)]
    if not with_gf:
        gf = None
    scale = 0.3
    f = orc.forward_kq(grid, kcube, q, k, v, gc, gf, topk, scale=scale, want_sc=True)
    idx = f["block_idx"]
    # the selection itself: the topk largest finite logits of each row, ascending
    for c in range(Nc):
        row = f["sc"][0, 1, c]
        assert np.array_equal(idx[0, 1, c], np.sort(np.argsort(-row, kind="stable")[:topk]))
    tq, tk, tv, tgc = (torch.from_numpy(x).requires_grad_(True) for x in (q, k, v, gc))
    tgf = torch.from_numpy(gf).requires_grad_(True) if with_gf else None
    out = torch_vsa_kq(grid, kcube, tq, tk, tv, tgc, tgf, idx, scale)
    assert np.abs(out.detach().numpy() - f["out"]).max() < 1e-12
    (out * torch.from_numpy(do)).sum().backward()
    b = orc.backward_kq(grid, kcube, q, k, v, gc, gf, do, idx, topk, scale=scale)
    vm = valid[None, None, :, None]
    assert np.abs(b["dq"] - tq.grad.numpy() * vm).max() < 1e-11
    assert np.abs(b["dk"] - tk.grad.numpy() * vm).max() < 1e-11
    assert np.abs(b["dv"] - tv.grad.numpy() * vm).max() < 1e-11
    assert np.abs(b["dgate_c"] - tgc.grad.numpy()).max() < 1e-11
    if with_gf:
        assert np.abs(b["dgate_f"] - tgf.grad.numpy()).max() < 1e-11


def test_paper_anchors():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_anchors.txt")
    gold = {}
    for line in open(path):
        line = line.split("#")[0].split()
        if len(line) == 2:
            gold[line[0]] = float(line[1])
    g = Grid(16, 32, 32)
    Np, Nc, Bk = g.dims()
    assert Bk == gold["tile_tokens"] and Nc == 256
    dense = orc.attention_flops(Np, Np, 128, 12)
    sparse = orc.attention_flops(Np, 32 * Bk, 128, 12)
    assert dense / sparse == gold["attention_flops_cut_k32_of_256"]
    assert 1 - 32 * Bk / Np == gold["sparsity_k32_of_256_cubes"]
    assert orc.attention_flops(Np, Np, 128, 12, with_backward=True) / dense == gold["fwd_bwd_over_fwd"]
    g2 = Grid(16, 28, 52)
    assert g2.Nc == gold["cubes_16x28x52"]
    assert abs((1 - 32 / g2.Nc) - gold["sparsity_16x28x52_k32"]) < 5e-4
    assert abs(100_000 / Bk - gold["cubes_for_100k_tokens"]) / gold["cubes_for_100k_tokens"] < 0.05
    coarse = orc.attention_flops(Nc, Nc, 128, 12)
    assert coarse / sparse < gold["coarse_flops_fraction_max"]

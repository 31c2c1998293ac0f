"""Video Sparse Attention as a differentiable PyTorch op (App. B: tile -> sparse attention -> untile).

Marshalling only: the token permutation, the forward and the backward all run in libvsa.so's
kernels; torch supplies device memory, the current stream and the autograd graph.  Tensors are in
the layout a video DiT holds them in, token-major raster order: bf16 [B, L, H, d] with
L = T*Hh*W and n = t*Hh*W + h*W + w (Sec. 2.1).

    out = video_sparse_attention(q, k, v, gate_c, gate_f, grid=(T, Hh, W), topk=K)

gate_f may be None (a fine gate of ones, Sec. 2.3).  No gradient flows through the top-K selection.
A model that keeps its activations in tiled order across layers (App. B caption) should call the
vsa_* entry points directly and skip the permutations.
"""
import torch

from . import vsa


class _VideoSparseAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, gate_c, gate_f, grid, topk, cube, softmax_scale, flags):
        B, L, H, d = q.shape
        T, Hh, W = grid
        assert L == T * Hh * W, "q is [B, T*Hh*W, H, d]"
        pb = vsa.Problem(B, H, T, Hh, W, d, topk, tuple(cube), float(softmax_scale or 0.0), int(flags))
        buf = vsa.Buffers(pb, device=q.device, backward=False)
        shape = (B, H, buf.Np, d)

        def tiled(x):
            y = torch.empty(shape, dtype=torch.bfloat16, device=q.device)
            vsa.vsa_tile_permute(pb, x.contiguous(), y, inverse=False, blhd=True)
            return y

        tq, tk, tv, tgc = tiled(q), tiled(k), tiled(v), tiled(gate_c)
        tgf = None if gate_f is None else tiled(gate_f)
        buf.forward(tq, tk, tv, tgc, tgf)
        out = torch.empty_like(q)
        vsa.vsa_tile_permute(pb, buf.out, out, inverse=True, blhd=True)
        ctx.pb, ctx.buf = pb, buf
        ctx.save_for_backward(tq, tk, tv, tgc, tgf)
        return out

    @staticmethod
    def backward(ctx, dout):
        pb, fw = ctx.pb, ctx.buf
        tq, tk, tv, tgc, tgf = ctx.saved_tensors
        shape = tq.shape
        tdo = torch.empty(shape, dtype=torch.bfloat16, device=tq.device)
        vsa.vsa_tile_permute(pb, dout.contiguous(), tdo, inverse=False, blhd=True)
        bw = vsa.Buffers(pb, device=tq.device, backward=True, with_gate_f=tgf is not None)
        vsa.vsa_backward(pb, tq, tk, tv, tgc, tgf, tdo, fw.block_idx, fw.out_fine, fw.lse_fine, fw.out_coarse,
                         fw.lse_coarse, bw.dq, bw.dk, bw.dv, bw.dgate_c, bw.dgate_f, bw.workspace)

        def raster(x):
            if x is None:
                return None
            y = torch.empty((pb.B, pb.T * pb.Hh * pb.W, pb.H, pb.d), dtype=torch.bfloat16, device=x.device)
            vsa.vsa_tile_permute(pb, x, y, inverse=True, blhd=True)
            return y

        return (raster(bw.dq), raster(bw.dk), raster(bw.dv), raster(bw.dgate_c), raster(bw.dgate_f),
                None, None, None, None, None)


def video_sparse_attention(q, k, v, gate_c, gate_f=None, *, grid, topk, cube=(4, 4, 4), softmax_scale=None, flags=0):
    """q, k, v, gate_c, gate_f (or None): bf16 [B, T*Hh*W, H, d] on the GPU; returns bf16 of the same shape."""
    return _VideoSparseAttention.apply(q, k, v, gate_c, gate_f, tuple(grid), int(topk), tuple(cube), softmax_scale, flags)

"""Thin ctypes binding over libvsa.so (the C ABI declared in include/vsa.h).

Argument marshalling only: torch supplies device memory and the current HIP stream, every
step of the path runs inside the library's kernels.  There is no CPU fallback: if the
library has not been built, importing `lib()` raises.
"""
import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvsa.so")

VSA_FLAG_INDICES_GIVEN = 1
VSA_FLAG_RASTER_BLHD = 2
VSA_FLAG_WORKSPACE_KEPT = 4
VSA_FLAG_COARSE_FUSED = 8
VSA_FLAG_COARSE_UNFUSED = 64
VSA_FLAG_OUT_TOKEN_MAJOR = 16
VSA_FLAG_SELECT_POOLED_2X2 = 32
VSA_FLAG_KEY_CUBES_16 = 128
STATUS = {0: "VSA_OK", -1: "VSA_ERR_NULL", -2: "VSA_ERR_BAD_ARG", -3: "VSA_ERR_UNSUPPORTED", -4: "VSA_ERR_ALIGN",
          -5: "VSA_ERR_WORKSPACE", -6: "VSA_ERR_HIP", -7: "VSA_ERR_SCRATCH_LIMIT"}
EXPORTS = ["vsa_padded_tokens", "vsa_workspace_bytes", "vsa_tile_permute", "vsa_forward", "vsa_backward",
           "vsa_status_string", "vsa_profile_begin", "vsa_profile_count", "vsa_profile_name", "vsa_profile_ms",
           "vsa_profile_end", "vsa_bench_mfma_rate", "vsa_forward_static", "vsa_static_scratch_bytes", "vsa_host_replay_lists"]


class VsaParams(C.Structure):
    _fields_ = [("B", C.c_int32), ("H", C.c_int32), ("T", C.c_int32), ("Hh", C.c_int32), ("W", C.c_int32),
                ("Ct", C.c_int32), ("Ch", C.c_int32), ("Cw", C.c_int32), ("d", C.c_int32), ("topk", C.c_int32),
                ("softmax_scale", C.c_float), ("flags", C.c_uint32)]


class VsaError(RuntimeError):
    def __init__(self, fn, status):
        self.status = status
        msg = lib().vsa_status_string(status).decode()
        super().__init__(f"{fn}: {STATUS.get(status, status)} ({msg})")


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2505_13389_amd.build` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp = C.c_void_p
        L.vsa_padded_tokens.argtypes = [C.POINTER(VsaParams), C.POINTER(C.c_int64), C.POINTER(C.c_int32)]
        L.vsa_padded_tokens.restype = C.c_int
        L.vsa_workspace_bytes.argtypes = [C.POINTER(VsaParams), C.c_int]
        L.vsa_workspace_bytes.restype = C.c_size_t
        L.vsa_tile_permute.argtypes = [C.POINTER(VsaParams), vp, vp, C.c_int, vp]
        L.vsa_tile_permute.restype = C.c_int
        L.vsa_forward.argtypes = [C.POINTER(VsaParams)] + [vp] * 12 + [C.c_size_t, vp]
        L.vsa_forward.restype = C.c_int
        L.vsa_forward_static.argtypes = [C.POINTER(VsaParams)] + [vp] * 12
        L.vsa_forward_static.restype = C.c_int
        L.vsa_static_scratch_bytes.argtypes = []
        L.vsa_static_scratch_bytes.restype = C.c_size_t
        L.vsa_host_replay_lists.argtypes = [C.POINTER(VsaParams), vp, vp]
        L.vsa_host_replay_lists.restype = C.c_int
        L.vsa_backward.argtypes = [C.POINTER(VsaParams)] + [vp] * 17 + [C.c_size_t, vp]
        L.vsa_backward.restype = C.c_int
        L.vsa_bench_mfma_rate.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_double), C.c_void_p]
        L.vsa_profile_begin.argtypes = [C.c_int]
        L.vsa_profile_name.argtypes = [C.c_int]
        L.vsa_profile_name.restype = C.c_char_p
        L.vsa_profile_ms.argtypes = [C.c_int]
        L.vsa_profile_ms.restype = C.c_float
        L.vsa_status_string.argtypes = [C.c_int]
        L.vsa_status_string.restype = C.c_char_p
        _lib = L
    return _lib


@dataclass
class Problem:
    """Shape of one call; mirrors vsa_params_t."""
    B: int
    H: int
    T: int
    Hh: int
    W: int
    d: int
    topk: int
    cube: tuple = (4, 4, 4)
    softmax_scale: float = 0.0
    flags: int = 0

    def params(self, flags=None):
        return VsaParams(self.B, self.H, self.T, self.Hh, self.W, self.cube[0], self.cube[1], self.cube[2], self.d,
                         self.topk, self.softmax_scale, self.flags if flags is None else flags)


def problem_of(wl, topk=None) -> Problem:
    """The call shape of a named workload (synth.Workload); `topk` overrides the workload's own."""
    return Problem(wl.B, wl.H, wl.T, wl.Hh, wl.W, wl.d, wl.topk if topk is None else topk, tuple(wl.cube))


def _p(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def vsa_padded_tokens(pb: Problem):
    Np, Nc = C.c_int64(), C.c_int32()
    rc = lib().vsa_padded_tokens(C.byref(pb.params()), C.byref(Np), C.byref(Nc))
    if rc:
        raise VsaError("vsa_padded_tokens", rc)
    return Np.value, Nc.value


def vsa_workspace_bytes(pb: Problem, backward: bool) -> int:
    return int(lib().vsa_workspace_bytes(C.byref(pb.params()), int(backward)))


def vsa_tile_permute(pb: Problem, src: torch.Tensor, dst: torch.Tensor, inverse: bool = False, blhd: bool = False):
    flags = pb.flags | (VSA_FLAG_RASTER_BLHD if blhd else 0)
    rc = lib().vsa_tile_permute(C.byref(pb.params(flags)), _p(src), _p(dst), int(inverse), _stream())
    if rc:
        raise VsaError("vsa_tile_permute", rc)


def vsa_forward(pb: Problem, q, k, v, gate_c, gate_f, out, block_idx, out_fine, lse_fine, out_coarse, lse_coarse,
                workspace, indices_given: bool = False):
    flags = pb.flags | (VSA_FLAG_INDICES_GIVEN if indices_given else 0)
    rc = lib().vsa_forward(C.byref(pb.params(flags)), _p(q), _p(k), _p(v), _p(gate_c), _p(gate_f), _p(out),
                           _p(block_idx), _p(out_fine), _p(lse_fine), _p(out_coarse), _p(lse_coarse), _p(workspace),
                           0 if workspace is None else workspace.numel() * workspace.element_size(), _stream())
    if rc:
        raise VsaError("vsa_forward", rc)


def vsa_forward_static(pb: Problem, q, k, v, gate_c, gate_f, out, block_idx, out_fine, lse_fine, out_coarse,
                       lse_coarse, indices_given: bool = False):
    """vsa_forward on the library's own static scratch buffer (no workspace, no allocation)."""
    flags = pb.flags | (VSA_FLAG_INDICES_GIVEN if indices_given else 0)
    rc = lib().vsa_forward_static(C.byref(pb.params(flags)), _p(q), _p(k), _p(v), _p(gate_c), _p(gate_f), _p(out),
                                  _p(block_idx), _p(out_fine), _p(lse_fine), _p(out_coarse), _p(lse_coarse),
                                  _stream())
    if rc:
        raise VsaError("vsa_forward_static", rc)


def vsa_backward(pb: Problem, q, k, v, gate_c, gate_f, dout, block_idx, out_fine, lse_fine, out_coarse, lse_coarse,
                 dq, dk, dv, dgate_c, dgate_f, workspace, workspace_kept: bool = False):
    flags = pb.flags | (VSA_FLAG_WORKSPACE_KEPT if workspace_kept else 0)
    rc = lib().vsa_backward(C.byref(pb.params(flags)), _p(q), _p(k), _p(v), _p(gate_c), _p(gate_f), _p(dout),
                            _p(block_idx), _p(out_fine), _p(lse_fine), _p(out_coarse), _p(lse_coarse), _p(dq), _p(dk),
                            _p(dv), _p(dgate_c), _p(dgate_f), _p(workspace),
                            0 if workspace is None else workspace.numel() * workspace.element_size(), _stream())
    if rc:
        raise VsaError("vsa_backward", rc)


class Buffers:
    """Convenience holder: allocates every output / saved tensor / workspace of a Problem once."""

    def __init__(self, pb: Problem, device="cuda", backward=True, with_gate_f=True):
        self.pb = pb
        Np, Nc = vsa_padded_tokens(pb)
        self.Np, self.Nc = Np, Nc
        bf = dict(dtype=torch.bfloat16, device=device)
        f32 = dict(dtype=torch.float32, device=device)
        shp = (pb.B, pb.H, Np, pb.d)
        self.out = torch.empty(shp, **bf)
        self.out_fine = torch.empty(shp, **bf)
        self.lse_fine = torch.empty((pb.B, pb.H, Np), **f32)
        self.out_coarse = torch.empty((pb.B, pb.H, Nc, pb.d), **f32)
        self.lse_coarse = torch.empty((pb.B, pb.H, Nc), **f32)
        rows = Nc // 4 if pb.flags & VSA_FLAG_SELECT_POOLED_2X2 else Nc  # that flag's lists are per tile of 4 cubes
        self.block_idx = torch.empty((pb.B, pb.H, rows, pb.topk), dtype=torch.int32, device=device)
        nbytes = max(vsa_workspace_bytes(pb, False), vsa_workspace_bytes(pb, True) if backward else 0)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
        if backward:
            self.dq, self.dk, self.dv = (torch.empty(shp, **bf) for _ in range(3))
            self.dgate_c = torch.empty(shp, **bf)
            self.dgate_f = torch.empty(shp, **bf) if with_gate_f else None

    def forward(self, q, k, v, gate_c, gate_f, indices_given=False):
        vsa_forward(self.pb, q, k, v, gate_c, gate_f, self.out, self.block_idx, self.out_fine, self.lse_fine,
                    self.out_coarse, self.lse_coarse, self.workspace, indices_given=indices_given)

    def backward(self, q, k, v, gate_c, gate_f, dout, workspace_kept=False):
        """workspace_kept: forward() ran on the same q, k, v and nothing touched the workspace since."""
        vsa_backward(self.pb, q, k, v, gate_c, gate_f, dout, self.block_idx, self.out_fine, self.lse_fine,
                     self.out_coarse, self.lse_coarse, self.dq, self.dk, self.dv, self.dgate_c, self.dgate_f,
                     self.workspace, workspace_kept=workspace_kept)


def vsa_host_replay_lists(pb: Problem, block_idx):
    """Host-only: replays the kernels' list index arithmetic on a numpy int32 [B,H,Nc,topk] array.
    Returns (status, report dict)."""
    import numpy as np
    idx = np.ascontiguousarray(block_idx, dtype=np.int32)
    rep = (C.c_int64 * 8)()
    rc = lib().vsa_host_replay_lists(C.byref(pb.params()), idx.ctypes.data_as(C.c_void_p), rep)
    names = ("violations", "longest_list", "items", "slots", "split_lists", "col_entries", "seg", "cap")
    return rc, dict(zip(names, (int(v) for v in rep)))


def vsa_bench_mfma_rate(operands: torch.Tensor, sink: torch.Tensor, workgroups: int, iters: int) -> float:
    """Enqueues the matrix-core rate probe on the current stream; returns the flops of the launch."""
    assert operands.numel() * operands.element_size() >= 65536 and sink.numel() >= workgroups * 256
    fl = C.c_double(0.0)
    rc = lib().vsa_bench_mfma_rate(_p(operands), _p(sink), workgroups, iters, C.byref(fl), _stream())
    if rc:
        raise VsaError("vsa_bench_mfma_rate", rc)
    return fl.value


def vsa_profile_begin(max_records: int):
    rc = lib().vsa_profile_begin(max_records)
    if rc:
        raise VsaError("vsa_profile_begin", rc)


def vsa_profile_end():
    """Synchronise first.  Returns [(kernel name, milliseconds)] in launch order and stops recording."""
    L = lib()
    recs = [(L.vsa_profile_name(i).decode(), float(L.vsa_profile_ms(i))) for i in range(L.vsa_profile_count())]
    L.vsa_profile_end()
    return recs

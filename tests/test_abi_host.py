"""Host-side checks of the C ABI (no GPU): the library loads, exports what the header declares,
and its host-only entry points and argument validation behave as documented."""
import ctypes as C
import os
import re

import pytest

from paper_2505_13389_amd import vsa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(vsa.LIB_PATH):
        from paper_2505_13389_amd import build
        build.build()
    return vsa.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "vsa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vsa_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(vsa.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_padded_tokens_and_workspace(lib):
    pb = vsa.Problem(1, 12, 21, 30, 52, 128, 78)
    assert vsa.vsa_padded_tokens(pb) == (39936, 624)
    assert vsa.vsa_padded_tokens(vsa.Problem(1, 40, 21, 45, 80, 128, 180)) == (92160, 1440)
    assert vsa.vsa_padded_tokens(vsa.Problem(1, 2, 8, 16, 16, 64, 8)) == (2048, 32)
    assert vsa.vsa_padded_tokens(vsa.Problem(1, 12, 21, 30, 52, 128, 39, cube=(4, 4, 8))) == (43008, 336)
    assert vsa.vsa_padded_tokens(vsa.Problem(1, 12, 21, 30, 52, 128, 20, cube=(4, 8, 8))) == (43008, 168)
    f, b = vsa.vsa_workspace_bytes(pb, False), vsa.vsa_workspace_bytes(pb, True)
    assert 0 < f < b
    assert f >= 3 * 12 * 624 * 128 * 4  # at least the three pooled tensors


@pytest.mark.parametrize("kwargs,status", [
    (dict(cube=(2, 2, 2)), -3), (dict(d=96), -3), (dict(T=0), -2), (dict(B=0), -2),
    (dict(T=256, Hh=256, W=256), -3),  # more cubes than VSA_MAX_CUBES
    (dict(softmax_scale=1e-3), -2),    # the pad-key bias would no longer mask
    (dict(cube=(4, 8, 16)), -3),       # 512-token cubes
])
def test_bad_parameters_are_rejected(lib, kwargs, status):
    base = dict(B=1, H=2, T=8, Hh=16, W=16, d=64, topk=8)
    base.update(kwargs)
    pb = vsa.Problem(**base)
    Np, Nc = C.c_int64(), C.c_int32()
    assert lib.vsa_padded_tokens(C.byref(pb.params()), C.byref(Np), C.byref(Nc)) == status
    assert vsa.vsa_workspace_bytes(pb, False) == 0


def test_null_and_topk_validation_happens_before_any_launch(lib):
    pb = vsa.Problem(1, 2, 8, 16, 16, 64, 8)
    assert lib.vsa_forward(C.byref(pb.params()), *([None] * 12), 0, None) == -1
    assert lib.vsa_backward(C.byref(pb.params()), *([None] * 17), 0, None) == -1
    assert lib.vsa_tile_permute(C.byref(pb.params()), None, None, 0, None) == -1
    assert lib.vsa_forward(None, *([None] * 12), 0, None) == -1
    bad = vsa.Problem(1, 2, 8, 16, 16, 64, 0)
    assert lib.vsa_forward(C.byref(bad.params()), *([None] * 12), 0, None) == -2
    assert vsa.vsa_workspace_bytes(vsa.Problem(1, 2, 8, 16, 16, 64, 33), False) == 0


def test_list_index_rules_with_tile_lists(lib):
    """Mismatched granularity: the lists name tiles of (1,2,2) cubes; hostile tile lists stay in bounds too."""
    import dataclasses
    import numpy as np
    pb = dataclasses.replace(vsa.Problem(1, 2, 8, 16, 32, 64, 5), flags=vsa.VSA_FLAG_SELECT_POOLED_2X2)
    _, Nc = vsa.vsa_padded_tokens(pb)
    Ns = Nc // 4
    rng = np.random.Generator(np.random.PCG64(3))
    hostile = rng.integers(-5, Ns + 5, size=(1, 2, Ns, 5), dtype=np.int64).astype(np.int32)
    hostile[0, 0, 0, :] = np.iinfo(np.int32).min
    for lists in (hostile, np.broadcast_to(np.arange(5, dtype=np.int32), (1, 2, Ns, 5))):
        rc, rep = vsa.vsa_host_replay_lists(pb, lists)
        assert rc == 0 and rep["violations"] == 0, rep
        assert rep["longest_list"] <= Nc and rep["col_entries"] <= Nc * 20


def test_key_cubes_16_parameter_checks(lib):
    """Key cubes of 16 tokens: topk counts LIVE key cubes; needs (4,4,4) cubes, no pooled selection, <= 4096 key cubes."""
    import dataclasses
    flag = vsa.VSA_FLAG_KEY_CUBES_16
    ok = dataclasses.replace(vsa.Problem(1, 1, 7, 14, 30, 64, 4 * 4 * 15), flags=flag)   # every live key cube of 256
    assert vsa.vsa_workspace_bytes(ok, True) > vsa.vsa_workspace_bytes(ok, False) > 0
    assert vsa.vsa_workspace_bytes(dataclasses.replace(ok, topk=4 * 4 * 15 + 1), False) == 0  # ... and a dead one
    big_cube = dataclasses.replace(vsa.Problem(1, 1, 8, 16, 32, 64, 2, cube=(4, 4, 8)), flags=flag)
    assert vsa.vsa_workspace_bytes(big_cube, False) == 0
    both = dataclasses.replace(vsa.Problem(1, 1, 8, 16, 32, 64, 2), flags=flag | vsa.VSA_FLAG_SELECT_POOLED_2X2)
    assert vsa.vsa_workspace_bytes(both, False) == 0
    assert vsa.vsa_workspace_bytes(dataclasses.replace(vsa.Problem(1, 1, 32, 32, 64, 64, 8), flags=flag), False) > 0  # 4096 key cubes
    assert vsa.vsa_workspace_bytes(dataclasses.replace(vsa.Problem(1, 1, 24, 48, 64, 64, 8), flags=flag), False) == 0  # 4608


def test_list_index_rules_with_key_cube_lists(lib):
    """Lists of key cubes of 16 tokens: hostile entries are clamped (fetches) or skipped (transposed map) against 4*Nc."""
    import dataclasses
    import numpy as np
    pb = dataclasses.replace(vsa.Problem(2, 2, 7, 14, 30, 64, 21), flags=vsa.VSA_FLAG_KEY_CUBES_16)
    _, Nc = vsa.vsa_padded_tokens(pb)
    rng = np.random.Generator(np.random.PCG64(5))
    hostile = rng.integers(-9, 4 * Nc + 9, size=(2, 2, Nc, 21), dtype=np.int64).astype(np.int32)
    hostile[0, 0, 0, :] = np.iinfo(np.int32).max
    hostile[1, 1, 1, :] = np.iinfo(np.int32).min
    same = np.broadcast_to(np.arange(21, dtype=np.int32) * 3, (2, 2, Nc, 21))
    for lists in (hostile, same):
        rc, rep = vsa.vsa_host_replay_lists(pb, lists)
        assert rc == 0 and rep["violations"] == 0, rep
        assert rep["longest_list"] <= Nc and rep["col_entries"] <= Nc * 21


def test_status_strings(lib):
    seen = set()
    for s in range(0, -8, -1):
        msg = lib.vsa_status_string(s)
        assert msg and msg not in seen
        seen.add(msg)
    assert lib.vsa_status_string(-99) == b"unknown status"


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: bench.py --gpus N>1 exits with a message before touching a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr
    assert r.stdout.strip() == ""


@pytest.mark.parametrize("shape,topk,cube", [((2, 2, 8, 16, 16), 8, (4, 4, 4)), ((1, 2, 12, 16, 20), 6, (4, 4, 4)),
                                             ((1, 1, 21, 30, 52), 78, (4, 4, 4)), ((1, 2, 16, 32, 32), 130, (4, 4, 4)),
                                             ((1, 2, 16, 32, 32), 9, (4, 4, 8)), ((2, 1, 12, 30, 30), 5, (4, 8, 8))])
def test_list_index_rules_keep_hostile_lists_in_bounds(lib, shape, topk, cube):
    """The clamp / skip / split arithmetic the kernels apply to block lists, replayed on the CPU through
    the same functions: lists full of out-of-range entries, duplicates and disorder, lists where every
    query cube names the same few key cubes (longest possible transposed lists), and ordinary ones."""
    import numpy as np
    B, H, T, Hh, W = shape
    pb = vsa.Problem(B, H, T, Hh, W, 64, topk, cube=cube)
    Np, Nc = vsa.vsa_padded_tokens(pb)
    m = cube[0] * cube[1] * cube[2] // 64  # attention blocks of 64 rows per cube: the kernels' lists name blocks
    rng = np.random.Generator(np.random.PCG64(17))
    hostile = rng.integers(-9, Nc + 9, size=(B, H, Nc, topk), dtype=np.int64).astype(np.int32)
    hostile[0, 0, 0, :] = np.iinfo(np.int32).max
    hostile[0, 0, 1 % Nc, :] = np.iinfo(np.int32).min
    same = np.broadcast_to(np.arange(topk, dtype=np.int32) % Nc, (B, H, Nc, topk))
    ordinary = np.sort(np.argsort(rng.random((B, H, Nc, Nc)), axis=-1)[..., :topk], axis=-1).astype(np.int32)
    for lists in (hostile, same, ordinary):
        rc, rep = vsa.vsa_host_replay_lists(pb, lists)
        assert rc == 0 and rep["violations"] == 0, rep
        assert rep["longest_list"] <= Nc * m and rep["col_entries"] <= Nc * m * topk * m
        assert rep["items"] <= Nc * m + rep["cap"] and rep["slots"] <= rep["cap"]
        assert rep["split_lists"] <= rep["cap"] // 2
    rc, rep = vsa.vsa_host_replay_lists(pb, same)
    assert rep["longest_list"] == Nc * m
    if Nc * m > rep["seg"] and 2 * topk * m <= rep["cap"]:  # (more equal long lists than slots: nothing to balance)
        assert rep["split_lists"] == topk * m and rep["items"] > Nc * m  # the sink lists are shared by several workgroups

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
    f, b = vsa.vsa_workspace_bytes(pb, False), vsa.vsa_workspace_bytes(pb, True)
    assert 0 < f < b
    assert f >= 3 * 12 * 624 * 128 * 4  # at least the three pooled tensors


@pytest.mark.parametrize("kwargs,status", [
    (dict(cube=(2, 2, 2)), -3), (dict(d=96), -3), (dict(T=0), -2), (dict(B=0), -2),
    (dict(T=256, Hh=256, W=256), -3),  # more cubes than VSA_MAX_CUBES
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

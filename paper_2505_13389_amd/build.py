"""Compiles the HIP sources under csrc/ into libvsa.so (gfx950 only), in-tree."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libvsa.so")
SOURCES = ["vsa_api.hip", "permute_pool.hip", "coarse.hip", "fine_fwd.hip", "bwd_small.hip", "fine_bwd.hip"]
# Packed-fp32 VALU forms are disabled on purpose (hipcc would otherwise emit them from plain float code).
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _compile(src: str, extra) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    r = subprocess.run(["hipcc", *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj], capture_output=True, text=True)
    # the host pass does not know the packed-fp32 feature and says so on every file: drop that line
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err[-4000:]}")
    if err.strip():
        print(err)
    return obj


def build(extra_flags=()) -> str:
    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(lambda s: _compile(s, list(extra_flags)), SOURCES))
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(sys.argv[1:]))

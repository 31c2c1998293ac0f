"""Builds the two shared objects of the CPU oracle (fp64 and fp32) with gcc.

Test infrastructure: only tests, the smoke check and the benchmark's CPU-baseline leg use it.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "vsa_oracle.c")


def lib_path(real: str) -> str:
    return os.path.join(HERE, f"libvsa_oracle_{real}.so")


def build(force: bool = False) -> None:
    for real, ctype in (("f64", "double"), ("f32", "float")):
        out = lib_path(real)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
            continue
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               f"-DREAL={ctype}", "-o", out, SRC, "-lm"]
        subprocess.run(cmd, check=True)


if __name__ == "__main__":
    build(force=True)
    print("built", lib_path("f64"), lib_path("f32"))

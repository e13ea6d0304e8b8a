"""Build the CPU oracle's shared libraries (TEST INFRASTRUCTURE, not product).

Two builds of the same source: liborc_f64.so (double; the parity reference) and
liborc_f32.so (float; the "plain fp32 CPU implementation" that is timed as the
CPU baseline).  g++ -O2 with OpenMP, no BLAS.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))


def lib_path(real: str) -> str:
    return os.path.join(HERE, f"liborc_{real}.so")


def build(force: bool = False) -> None:
    src = os.path.join(HERE, "orc_ops.cpp")
    for real, ctype in (("f64", "double"), ("f32", "float")):
        out = lib_path(real)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(src):
            continue
        cmd = ["g++", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c++17",
               f"-DORC_REAL={ctype}", "-o", out, src]
        subprocess.check_call(cmd)


if __name__ == "__main__":
    build(force="--force" in sys.argv)
    print("oracle built:", lib_path("f64"), lib_path("f32"))

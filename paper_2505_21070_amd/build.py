"""Builds libdualparal.so for gfx950 with hipcc (in-tree, next to this file)."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdualparal.so")
SOURCES = ["stage.hip", "schedule.cpp", "elementwise.hip", "gemm_f32.hip", "attn_f32.hip", "gemm_bf16.hip", "attn_bf16.hip", "probe.hip", "ends.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wno-unused-value",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = False) -> str:
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(objdir, src + ".o")
        cmd = ["hipcc", *FLAGS, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{r.stderr}")
        if verbose:
            print("compiled", src)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    return LIB


def is_stale() -> bool:
    """True when no library is there or a source or header is newer than it."""
    if not os.path.exists(LIB):
        return True
    built = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    deps.append(os.path.join(os.path.dirname(HERE), "include", "dualparal.h"))
    return any(os.path.getmtime(d) > built for d in deps if os.path.isfile(d))


def ensure_built() -> str:
    """For the scripts around the library (tests, bench, smoke): loads what is built, and builds only if no
    library is there or a source is newer than it (so a stale binary is never tested).  The binding never
    calls this; without a library it raises."""
    return build() if is_stale() else LIB


if __name__ == "__main__":
    print(build(verbose=True))

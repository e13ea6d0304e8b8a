"""Size arithmetic of the stage and model-ends configuration code under UndefinedBehaviorSanitizer: the two
source files with that host logic are rebuilt with trapping checks on the host side only (the device code is
untouched and never runs), linked with the library's other objects, and a child process feeds
dp_stage_workspace_bytes / dp_ends_workspace_bytes extreme configurations (tests/host_config_fuzz.py)."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2505_21070_amd")
sys.path.insert(0, ROOT)


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_config_size_arithmetic_under_ubsan(tmp_path):
    from paper_2505_21070_amd import build as B
    checked = ("stage.hip", "ends.hip")
    san = ["-Xarch_host", "-fsanitize=signed-integer-overflow,shift,integer-divide-by-zero,bounds,null,pointer-overflow",
           "-Xarch_host", "-fsanitize-trap=all"]
    objs = []
    for src in B.SOURCES:
        path = os.path.join(B.CSRC, src)
        built = os.path.join(PKG, "_build", src + ".o")
        if src not in checked and os.path.exists(built) and os.path.getmtime(built) >= os.path.getmtime(path):
            objs.append(built)                 # kernels only: reuse the library's own object
            continue
        obj = str(tmp_path / (src + ".o"))
        flags = [f for f in B.FLAGS if f != "-O3"] + ["-O1"] + (san if src in checked else [])
        subprocess.run(["hipcc", *flags, "-x", "hip", "-c", path, "-o", obj], check=True, capture_output=True, text=True)
        objs.append(obj)
    lib = str(tmp_path / "libdualparal_ubsan.so")
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs], check=True,
                   capture_output=True, text=True)
    r = subprocess.run([sys.executable, os.path.join(ROOT, "tests", "host_config_fuzz.py"), lib], capture_output=True,
                       text=True, timeout=600)
    tail = r.stdout.strip().splitlines()[-2:]
    assert r.returncode == 0, (r.returncode, tail, r.stderr[-2000:])
    assert tail[-1].startswith("ok "), tail

"""include/dualparal.h from a C compiler: strict C99 compile of a client (tests/c_abi_client.c), linked against
the built library, running the host-only calls (no GPU needed)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2505_21070_amd")


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_c99_client_links_and_runs(tmp_path):
    assert os.path.exists(os.path.join(PKG, "libdualparal.so")), "build the library first (paper_2505_21070_amd/build.py)"
    exe = str(tmp_path / "c_abi_client")
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c_abi_client.c"), "-L", PKG, "-ldualparal", f"-Wl,-rpath,{PKG}",
           "-Wl,-rpath,/opt/rocm/lib", "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr[-2000:])
    assert r.stdout.startswith("ok ") and abs(float(r.stdout.split()[1]) - 11 / 211) < 1e-6

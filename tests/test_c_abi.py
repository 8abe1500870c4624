"""The boundary is a C ABI: a plain C99 program includes include/th.h, links the library and
drives a host-only plan through it (no GPU, no Python in the call path)."""
import os
import shutil
import subprocess

import pytest

import paper_2604_09107_amd as th

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_plain_c_caller(tmp_path):
    libdir = os.path.dirname(th.library_path())
    exe = str(tmp_path / "abi_host")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror",
                           "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "c", "abi_host.c"),
                           "-o", exe, "-L", libdir, "-ltensorhub_reshard",
                           "-Wl,-rpath," + libdir, "-Wl,-rpath," + os.path.join(rocm, "lib")])
    out = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert out.returncode == 0, out.stderr
    assert "c abi ok" in out.stdout

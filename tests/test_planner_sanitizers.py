"""The host planner under AddressSanitizer and UndefinedBehaviorSanitizer: tests/c/planner_host.cpp
is compiled together with th_layouts.cpp and th_planner.cpp (host code only, no HIP), plans the
full-size workloads and thousands of odd explicit segments, compares one planner thread with three,
and makes every allocation of a plan fail in turn."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2604_09107_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_planner_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "planner_host")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-Werror",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                           os.path.join(ROOT, "tests", "c", "planner_host.cpp"),
                           os.path.join(CSRC, "th_layouts.cpp"), os.path.join(CSRC, "th_planner.cpp"),
                           "-o", exe, "-pthread"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:allocator_may_return_null=1:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    out = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-4000:]
    assert "planner host ok" in out.stdout

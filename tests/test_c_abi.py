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


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_allocation_failures_never_cross_the_boundary(tmp_path):
    """Every allocation inside th_plan_create / th_plan_create_from_segments (host-only plans) fails
    in turn: the call returns TH_ERR_NOMEM with a message, or TH_OK when the failure hit nothing."""
    libdir = os.path.dirname(th.library_path())
    exe = str(tmp_path / "abi_nomem")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-Wall", "-Wextra", "-Werror", "-Wno-mismatched-new-delete",
                           "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "c", "abi_nomem.cpp"),
                           "-o", exe, "-L", libdir, "-ltensorhub_reshard",
                           "-Wl,-rpath," + libdir, "-Wl,-rpath," + os.path.join(rocm, "lib")])
    out = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "c abi nomem ok" in out.stdout


def test_one_planner_thread_builds_the_same_lists():
    """TH_CFG_PLANNER_THREADS = 1 (what a plan falls back to when a thread cannot be started) against
    the default three threads, on a plan large enough for the threaded build."""
    import numpy as np
    n = 3000
    segs = np.zeros(n, dtype=th.binding.SEGMENT_NP)
    segs["src_tensor"] = np.arange(n)
    segs["nrows"], segs["row_len"] = 40, 100 + np.arange(n) % 20
    segs["src_row_stride"], segs["dst_row_stride"] = 125, 120
    segs["dst_elem_off"] = np.arange(n) * 5000
    segs["src_dtype"], segs["dst_dtype"] = th.TH_F32, th.TH_BF16
    lists = []
    assert th.th_config_get(th.TH_CFG_PLANNER_THREADS) == 3
    try:
        for threads in (3, 1):
            th.th_config_set(th.TH_CFG_PLANNER_THREADS, threads)
            plan = th.th_plan_create_from_segments(segs, np.full(n, 5000), [n * 5000], 1 << 20, th.TH_FLAG_HOST_ONLY)
            assert plan.num_tiles(0) >= 4096
            lists.append([[bytes(plan.tile(side, i)) for i in range(plan.num_tiles(side))] for side in range(3)])
            plan.destroy()
    finally:
        th.th_config_set(th.TH_CFG_PLANNER_THREADS, 3)
    assert lists[0] == lists[1]
    with pytest.raises(th.ThError):
        th.th_config_set(th.TH_CFG_PLANNER_THREADS, 0)

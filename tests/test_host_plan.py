"""The host side of the library that does pointer arithmetic on the slab (make_plan, build_work_list,
make_refresh_plan in csrc/fira_plan.h) built on its own with the address and undefined-behaviour sanitizers
and fuzzed with random descriptor lists (tests/host_plan_check.cpp): odd n, r = 1, r = min(m, n), ld > n, mixed
dtypes, 1 to 1024 matrices.  Every piece must be aligned, inside the total and disjoint; every tile grid covered
exactly once; no write outside the work-list block.  CPU only."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "host_plan_check.cpp")
# on a hipcc line each -fsanitize= option follows an -Xarch_host, so that only the host code is instrumented
FLAGS = ["-x", "hip", "--cuda-host-only", "-std=c++17", "-O1", "-g", "-Xarch_host", "-fsanitize=address",
         "-Xarch_host", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]


def _build(tmp_path, name, extra=()):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    exe = str(tmp_path / name)
    res = subprocess.run([hipcc, *FLAGS, *extra, SRC, "-o", exe], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    return exe


def test_planner_under_the_sanitizers(tmp_path):
    exe = _build(tmp_path, "host_plan_check")
    res = subprocess.run([exe, "400"], capture_output=True, text=True, timeout=600)
    print(res.stdout[-2000:], res.stderr[-2000:])
    assert res.returncode == 0, (res.stdout[-3000:], res.stderr[-3000:])
    assert "0 failure(s)" in res.stdout


def test_the_check_sees_a_write_past_the_work_list(tmp_path):
    """The same program with a work-list block that is too small: AddressSanitizer must stop it."""
    exe = _build(tmp_path, "host_plan_check_short", ["-DFIRA_PLAN_CHECK_SHORT_STAGE"])
    res = subprocess.run([exe, "50"], capture_output=True, text=True, timeout=600)
    assert res.returncode != 0 and "AddressSanitizer" in res.stderr and "heap-buffer-overflow" in res.stderr

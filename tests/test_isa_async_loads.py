"""The projection kernels (plain, and fused with Adam) request their gradient tiles with inline-assembly
loads and wait for them with explicit queue depths.  This compiles the device code to assembly (no GPU needed) and checks that
the compiler never touches a register between such a load and the wait that covers it."""
import os
import shutil
import subprocess

import pytest

from paper_2410_01623_amd import build
import isa_async_check


def test_registers_of_asynchronous_loads_are_untouched_until_their_wait(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    out = tmp_path / "fira.s"
    flags = [f for f in build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [hipcc, *flags, "--cuda-device-only", "-S", os.path.join(build.CSRC, "fira.hip"), "-o", str(out)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    ks = {k: v for k, v in isa_async_check.kernels(out.read_text()).items() if "fira_project" in k}
    assert len(ks) == 4, list(ks)   # fira_project_kernel, fira_project_small_kernel, fira_project_adam_kernel<1>, <2>
    for name, body in ks.items():
        n, loads, viol = isa_async_check.check_kernel(body)
        assert loads >= 8, f"{name}: expected the pipelined loads, found {loads}"
        assert not viol, f"{name}: {len(viol)} instruction(s) touch a pending register, e.g. {viol[:3]}"


def test_checker_flags_a_planted_violation():
    body = """
	;;#ASMSTART
	global_load_dwordx4 v[10:13], v1, s[2:3]
	;;#ASMEND
	v_mov_b32_e32 v20, v11
	;;#ASMSTART
	s_waitcnt vmcnt(0) ; v[10:13]
	;;#ASMEND
	v_mov_b32_e32 v21, v12
	s_endpgm
"""
    n, loads, viol = isa_async_check.check_kernel(body)
    assert loads == 1 and len(viol) == 1 and "v20" in viol[0][1]

"""The boundary is a C ABI: include/gspmd.h must compile as plain C99 and the library must be usable from a C program
(host-only entry points here, so no GPU is needed)."""
import os
import subprocess

import paper_2105_04663_amd as g

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_is_c99_and_host_entry_points_work_from_c(tmp_path):
    lib = g.library_path()
    assert os.path.exists(lib)
    exe = str(tmp_path / "c_abi_check")
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c_abi_check.c"), "-o", exe, lib, "-Wl,-rpath," + os.path.dirname(lib)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, (run.returncode, run.stdout, run.stderr)
    assert "c abi ok" in run.stdout

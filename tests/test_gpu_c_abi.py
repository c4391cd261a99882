"""The C ABI used from a plain C99 program on the GPU: tests/c_device_check.c runs config 1 (the tiny 1-D sharded
matmul) through gspmd_shard_bounds / gspmd_shard_extract / gspmd_local_dot / gspmd_shard_assemble with HIP's C API for
the memory, and its reassembled product is compared with the oracle here."""
import os
import subprocess

import numpy as np
import pytest

import paper_2105_04663_amd as g
import workloads as wl
from oracle import dot as od

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_config1_from_a_c_program(tmp_path):
    lib = g.library_path()
    exe = str(tmp_path / "c_device_check")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(rocm, "include"), os.path.join(ROOT, "tests", "c_device_check.c"), "-o", exe, lib,
           "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-Wl,-rpath," + os.path.dirname(lib), "-Wl,-rpath," + os.path.join(rocm, "lib")]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    w = wl.tiny_1d()
    a, b = w.draw_lhs(), w.draw_rhs()
    fin, fout = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(fin, "wb") as f:
        f.write(a.astype(np.float32).tobytes())
        f.write(b.astype(np.float32).tobytes())
    run = subprocess.run([exe, fin, fout], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0 and "c device ok" in run.stdout, (run.returncode, run.stdout, run.stderr)
    got = np.fromfile(fout, dtype=np.float32).reshape(8, 90).astype(np.float64)
    ref = od.dot_general(a.astype(np.float64), b.astype(np.float64), (), (), (1,), (0,))
    assert np.isfinite(got).all()
    s, f = od.error_metrics(got, ref)
    assert s <= 1e-2 and f <= 1e-5, (s, f)

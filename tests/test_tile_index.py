"""CPU check of the MFMA kernel's index math (csrc/tile_index.h): tests/tile_index_check.hip is compiled with hipcc
and run on the host.  It replays tile loads and fragment reads for every tile format and checks that each lane
receives the operand elements the matrix instruction expects, that no load leaves the valid extents, and that the
tile order is a permutation."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_loads_fragment_reads_and_tile_order(tmp_path):
    exe = str(tmp_path / "tile_index_check")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    build = subprocess.run([hipcc, "--offload-arch=gfx950", "-O1", "-std=c++17", "-Wno-unused-command-line-argument",
                            "-x", "hip", os.path.join(ROOT, "tests", "tile_index_check.hip"), "-o", exe],
                           capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    run = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    assert run.returncode == 0 and "tile index ok" in run.stdout, run.stdout[-3000:] + run.stderr[-1000:]

"""Host code of the library (planner, transfer scheduler, tile tables) built with ASan + UBSan and checked on the
CPU: every tile the kernels will be given stays in bounds and the tables cover every element
exactly once.  No GPU, no HIP runtime."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2004_14020_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_planner_and_tile_tables_under_sanitizers(tmp_path):
    exe = str(tmp_path / "tiles_check")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(ROOT, "tests", "host", "tiles_check.cpp"),
           os.path.join(CSRC, "plan.cpp"), os.path.join(CSRC, "schedule.cpp"), os.path.join(CSRC, "tiles.cpp"),
           "-o", exe]
    subprocess.run(cmd, check=True)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-2000:]
    assert "tiles_check ok" in res.stdout

"""Host logic: the planner and decoder of the XCD-aware workgroup order
(csrc/tile_order.h), checked exhaustively on the CPU."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_every_row_tile_pair_is_decoded_exactly_once(tmp_path):
    if shutil.which("g++") is None:
        pytest.skip("g++ not available")
    exe = str(tmp_path / "tile_order_check")
    subprocess.run(["g++", "-O2", "-std=c++17", "-Wall", "-Wextra",
                    "-I", os.path.join(ROOT, "paper_2009_03816_amd", "csrc"),
                    os.path.join(HERE, "tile_order_check.cpp"), "-o", exe], check=True)
    run = subprocess.run([exe], capture_output=True, text=True)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "tile order ok" in run.stdout

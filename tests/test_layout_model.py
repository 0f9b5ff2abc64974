"""Host-side functional model of the bf16 kernel's LDS data path: compiled with g++ from the very
header the kernel uses (csrc/bf16_layout.h) and run on the CPU."""
import os
import subprocess


def test_lds_layout_model(tmp_path):
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = str(tmp_path / "layout_check")
    subprocess.run(["g++", "-std=c++17", "-O1", "-o", exe, os.path.join(root, "tests", "layout_check.cpp")],
                   check=True)
    res = subprocess.run([exe], capture_output=True, text=True)
    assert res.returncode == 0, res.stdout[-2000:]
    assert "layout checks passed" in res.stdout

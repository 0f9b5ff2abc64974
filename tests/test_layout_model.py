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


def test_symmetric_kernel_layout_model(tmp_path):
    """The same for the symmetric-operand kernel (csrc/symm_layout.h): slab map, the image read along and
    across its rows, the small operand's fragments, and the bookkeeping of super-tiles and terms."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = str(tmp_path / "symm_layout_check")
    subprocess.run(["g++", "-std=c++17", "-O1", "-o", exe, os.path.join(root, "tests", "symm_layout_check.cpp")],
                   check=True)
    res = subprocess.run([exe], capture_output=True, text=True)
    assert res.returncode == 0, res.stdout[-2000:]
    assert "symmetric layout checks passed" in res.stdout


def test_skinny_kernel_layout_model(tmp_path):
    """The same for the tall-skinny kernel (csrc/skinny_layout.h)."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = str(tmp_path / "skinny_layout_check")
    subprocess.run(["g++", "-std=c++17", "-O1", "-o", exe, os.path.join(root, "tests", "skinny_layout_check.cpp")],
                   check=True)
    res = subprocess.run([exe], capture_output=True, text=True)
    assert res.returncode == 0, res.stdout[-2000:]
    assert "skinny layout checks passed" in res.stdout


def test_conv_rows_kernel_layout_model(tmp_path):
    """The same for the few-channel convolution kernel (csrc/conv_rows_layout.h): staged rows, shifted and
    masked fragments, the matrix instruction's lanes and the channel map, against the definition."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = str(tmp_path / "conv_rows_layout_check")
    subprocess.run(["g++", "-std=c++17", "-O1", "-o", exe, os.path.join(root, "tests", "conv_rows_layout_check.cpp")],
                   check=True)
    res = subprocess.run([exe], capture_output=True, text=True)
    assert res.returncode == 0, res.stdout[-2000:]
    assert "conv rows layout checks passed" in res.stdout


def test_conv_halo_kernel_layout_model(tmp_path):
    """The same for the halo-staged 3 x 3 convolution kernel (csrc/conv_halo_layout.h): the staged input rows, every
    tap's fragments against the definition of the gather, bank groups, and the plan's cuts against a simulation."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = str(tmp_path / "conv_halo_layout_check")
    subprocess.run(["g++", "-std=c++17", "-O1", "-o", exe, os.path.join(root, "tests", "conv_halo_layout_check.cpp")],
                   check=True)
    res = subprocess.run([exe], capture_output=True, text=True)
    assert res.returncode == 0, res.stdout[-2000:]
    assert "conv halo layout checks passed" in res.stdout

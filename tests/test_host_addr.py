"""The per-tile index arithmetic of the GEMM kernels (csrc/lpg_addr.h) against its plain
definitions, on the host: reciprocal division, the tile walk, and the wave-uniform + per-lane
split of a staged fragment's source address (tests/host/addr_check.cpp)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_index_arithmetic_equals_its_definitions(tmp_path):
    exe = str(tmp_path / "addr_check")
    subprocess.run(["g++", "-O2", "-std=c++17", "-Wall", "-Wextra", "-Werror",
                    "-I", os.path.join(ROOT, "paper_2604_04599_amd", "csrc"),
                    "-o", exe, os.path.join(HERE, "host", "addr_check.cpp")], check=True)
    done = subprocess.run([exe], capture_output=True, text=True)
    assert done.returncode == 0, done.stdout + done.stderr
    assert done.stdout.startswith("ok ")

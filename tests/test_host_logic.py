"""Builds and runs the C++ test of the library's host-only bookkeeping (no GPU, no HIP)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_range_allocator_and_residency(tmp_path):
    exe = tmp_path / "host_logic_test"
    src = os.path.join(ROOT, "tests", "host_logic_test.cpp")
    inc = os.path.join(ROOT, "paper_2306_13835_amd", "csrc")
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-I", inc,
                    "-I", os.path.join(ROOT, "include"), src, "-o", str(exe)], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "host logic ok" in r.stdout

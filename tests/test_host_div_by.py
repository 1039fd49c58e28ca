"""Host logic: the launch-time division constants the matrix-core kernel's prologue uses
(csrc/div_by.h) give floor(n / d) for every 0 <= n < 2^31.  Compiled for the host with g++ and run
here; no GPU involved."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_div_by_matches_integer_division(tmp_path):
    exe = str(tmp_path / "div_by_check")
    subprocess.run(["g++", "-O2", "-std=c++17", "-I", os.path.join(ROOT, "paper_2010_00704_amd", "csrc"),
                    os.path.join(ROOT, "tests", "host", "div_by_check.cpp"), "-o", exe], check=True)
    out = subprocess.run([exe], stdout=subprocess.PIPE, text=True, timeout=300)
    assert out.returncode == 0, out.stdout
    assert out.stdout.strip() == "mismatches: 0"

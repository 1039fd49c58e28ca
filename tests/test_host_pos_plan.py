"""Host logic: the position-major tiling plan of the fused 3x3 convolution (csrc/pos_plan.h).  The
checker (tests/host/pos_plan_check.cpp) walks every tile of some fifteen thousand shapes through the
decode functions the kernel itself uses: every output pixel exactly once, no tap with real data left
out, tile counts, refusals.  Compiled for the host with g++ and run here; no GPU involved."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_position_major_plan_covers_every_pixel_once(tmp_path):
    exe = str(tmp_path / "pos_plan_check")
    subprocess.run(["g++", "-O2", "-std=c++17", "-I", os.path.join(ROOT, "paper_2010_00704_amd", "csrc"),
                    os.path.join(ROOT, "tests", "host", "pos_plan_check.cpp"), "-o", exe], check=True)
    out = subprocess.run([exe], stdout=subprocess.PIPE, text=True, timeout=300)
    assert out.returncode == 0, out.stdout
    assert "mismatches: 0" in out.stdout

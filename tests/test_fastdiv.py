"""The kernels' division by run-time constants (csrc/fastdiv.h) is exact over the whole 32-bit range:
compiled for the host and compared with the machine's integer division (no GPU)."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_fastdiv_is_exact_for_every_32_bit_dividend(tmp_path):
    exe = str(tmp_path / "fastdiv_check")
    subprocess.run(["g++", "-O2", "-std=c++17", "-I", os.path.join(ROOT, "paper_1603_05279_amd", "csrc"),
                    os.path.join(ROOT, "tests", "fastdiv_check.cpp"), "-o", exe], check=True)
    r = subprocess.run([exe], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout
    assert "mismatches 0" in r.stdout
    # the uncorrected multiply-high form is one too large on these (the reason for the correction step)
    assert "image 1 (uncorrected form: 2)" in r.stdout

"""Host-side checks of the GPU path's arithmetic building blocks, compiled for the CPU."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_selection_network_and_reciprocal_division(tmp_path):
    exe = str(tmp_path / "host_arith_check")
    subprocess.check_call(["g++", "-std=c++17", "-O2", "-mfma", "-ffp-contract=off",
                           "-I", os.path.join(ROOT, "paper_2202_07471_amd", "csrc"),
                           os.path.join(ROOT, "tests", "host_arith_check.cpp"), "-o", exe])
    out = subprocess.run([exe, "20000000"], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "network_mismatches=0" in out.stdout and "division_mismatches=0" in out.stdout

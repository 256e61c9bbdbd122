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


def test_reciprocal_division_is_exact_on_every_near_midpoint_case(tmp_path):
    """Proof by enumeration that the GPU path's three-operation division equals IEEE division
    (the argument is in the header of host_div_exhaustive.cpp)."""
    exe = str(tmp_path / "host_div_exhaustive")
    subprocess.check_call(["g++", "-std=c++17", "-O2", "-mfma", "-ffp-contract=off", "-fopenmp",
                           "-I", os.path.join(ROOT, "paper_2202_07471_amd", "csrc"),
                           os.path.join(ROOT, "tests", "host_div_exhaustive.cpp"), "-o", exe])
    out = subprocess.run([exe], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "mismatches=0" in out.stdout
    cases = int(out.stdout.split("near_midpoint_cases=")[1].split()[0])
    assert cases > 60_000_000


def test_variant_choice_covers_every_shape(tmp_path):
    exe = str(tmp_path / "host_plan_check")
    subprocess.check_call(["g++", "-std=c++17", "-O2",
                           "-I", os.path.join(ROOT, "paper_2202_07471_amd", "csrc"),
                           os.path.join(ROOT, "tests", "host_plan_check.cpp"), "-o", exe])
    out = subprocess.run([exe], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "plan_mismatches=0" in out.stdout


def test_reference_solver_under_sanitizers(tmp_path):
    """The CPU reference, compiled with the address and undefined-behaviour sanitizers, over
    assorted shapes, value patterns, modes and bit widths: nothing out of bounds, no overflow."""
    exe = str(tmp_path / "oracle_sanitize")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-static-libasan", "-pthread",
                           os.path.join(ROOT, "tests", "host_oracle_sanitize.cpp"), "-o", exe])
    out = subprocess.run([exe], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "sanitized_runs=1008" in out.stdout

"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, no device code involved).

Two small programs are compiled with gcc's -fsanitize=address,undefined and run:
  tests/sanitize/oracle_main.c   every entry point of the CPU oracle on exactly sized heap arrays;
  tests/sanitize/host_main.cpp   the HIP library's host-side table construction and launch planning
                                 (csrc/dq8_tables.cpp, dq8_plan.hpp, dq8_units.hpp), with element counts
                                 on both sides of 2^32.
A report from either sanitizer aborts the program, which fails the test.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-Wall", "-Wextra", "-Werror"]


def _run(cmd, exe):
    subprocess.check_call(cmd)
    # the link-order check is off so that a library preloaded into every process of the machine does not stop the run
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    p = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert p.returncode == 0, p.stdout[-2000:] + p.stderr[-4000:]
    assert "runtime error" not in p.stderr and "AddressSanitizer" not in p.stderr, p.stderr[-4000:]
    return p.stdout


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_main")
    out = _run(["gcc"] + SAN + ["-fno-fast-math", "-ffp-contract=off", "-fopenmp",
                                os.path.join(ROOT, "tests", "sanitize", "oracle_main.c"),
                                os.path.join(ROOT, "oracle", "dq8_oracle.c"), "-lm", "-o", exe], exe)
    assert "oracle checks ok" in out


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_tables_and_launch_plan_under_sanitizers(tmp_path):
    exe = str(tmp_path / "host_main")
    csrc = os.path.join(ROOT, "paper_1511_04561_amd", "csrc")
    out = _run(["g++", "-std=c++17"] + SAN + ["-I", os.path.join(ROOT, "include"), "-I", csrc,
                                             os.path.join(ROOT, "tests", "sanitize", "host_main.cpp"),
                                             os.path.join(csrc, "dq8_tables.cpp"), "-o", exe], exe)
    assert "host checks ok" in out

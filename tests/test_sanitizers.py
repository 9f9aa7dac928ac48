"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the CPU side: the oracle (all of
oracle/nm_oracle.c) and the library's host-side table code (csrc/nm_tables.cpp: descriptor
validation, chord / Algorithm 3 / Algorithm 2 builder, error paths of the table objects).  Each is
compiled for the host with -fsanitize=address,undefined together with a driver that calls every
entry point on small ragged inputs held in exactly sized heap buffers, and run as a program of its
own (no GPU, nothing preloaded)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]


def _run(cmd, exe):
    build = subprocess.run(cmd, capture_output=True, text=True, cwd=ROOT)
    assert build.returncode == 0, build.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0 and "SANITIZE_OK" in run.stdout, (run.stdout[-2000:], run.stderr[-4000:])
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr[-4000:]


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
def test_oracle_under_address_and_undefined_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    _run(["gcc", "-std=c11", *SAN, "-ffp-contract=off", "-fopenmp", "tests/sanitize/oracle_driver.c", "-o", exe, "-lm"], exe)


@pytest.mark.skipif(shutil.which("g++") is None or not os.path.exists("/opt/rocm/include/hip/hip_runtime.h"),
                    reason="g++ or the HIP headers not available")
def test_library_host_table_code_under_sanitizers(tmp_path):
    exe = str(tmp_path / "host_driver")
    _run(["g++", "-std=c++17", *SAN, "-D__HIP_PLATFORM_AMD__", "-I", "include", "-I", "paper_2305_14405_amd/csrc",
          "-I", "/opt/rocm/include", "tests/sanitize/host_driver.cpp", "paper_2305_14405_amd/csrc/nm_tables.cpp",
          "-o", exe, "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"], exe)

"""CPU build of the C oracle and of the host layer of the library (api.cpp, budget.cpp; kernel
launchers replaced by the checking stand-ins of tests/host_stubs.cpp) under AddressSanitizer and
UndefinedBehaviorSanitizer, driven by tests/sanitized_driver.py in a child process.  No GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fPIC", "-shared"]


def test_oracle_and_host_layer_are_clean_under_asan_and_ubsan(tmp_path):
    oracle_lib = str(tmp_path / "libvscan_oracle_san.so")
    host_lib = str(tmp_path / "libvscan_host_san.so")
    subprocess.check_call(["gcc", *SAN, "-fopenmp", "-Wall", "-Wextra", "-o", oracle_lib,
                           os.path.join(ROOT, "oracle", "vscan_oracle.c"), "-lm"])
    csrc = os.path.join(ROOT, "paper_2505_22654_amd", "csrc")
    subprocess.check_call(["g++", *SAN, "-std=c++17", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
                           "-Wno-unused-result", "-Wno-deprecated-declarations",
                           os.path.join(csrc, "api.cpp"), os.path.join(csrc, "budget.cpp"),
                           os.path.join(ROOT, "tests", "host_stubs.cpp"), "-o", host_lib,
                           "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"])
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    env = dict(os.environ, LD_PRELOAD=asan, PYTHONPATH=ROOT, OMP_NUM_THREADS="4",
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:exitcode=23",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1:exitcode=24")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "tests", "sanitized_driver.py"), oracle_lib,
                        host_lib], env=env, cwd=ROOT, capture_output=True, text=True, timeout=600)
    tail = (r.stdout + "\n" + r.stderr)[-4000:]
    assert r.returncode == 0, tail
    assert "sanitized-ok" in r.stdout, tail
    for marker in ("AddressSanitizer", "runtime error", "host_stubs:"):
        assert marker not in r.stderr, tail

"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

The oracle is the reference every GPU result is compared with, so its own memory accesses and
arithmetic are checked too: tests/asan_driver.cpp compiles the oracle's source into one executable
with -fsanitize=address,undefined and runs it on the tiny configuration and on the edge rows of the
parity tests (rows without mass, NaN and infinite entries, ragged and one-entry rows, empty list
slots, both forms of Algorithm 2's loop, the binned selection with and without shared race times).
"""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "asan_driver"
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fno-fast-math", "-ffp-contract=off", "-fopenmp",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
                    os.path.join(ROOT, "tests", "asan_driver.cpp"), "-o", str(exe)], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", OMP_NUM_THREADS="2")
    out = subprocess.run([str(exe)], capture_output=True, text=True, env=env)
    assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-4000:]
    assert "sanitizer run clean" in out.stdout
    assert "ERROR" not in out.stderr and "runtime error" not in out.stderr, out.stderr[-4000:]

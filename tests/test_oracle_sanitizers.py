"""The CPU oracle under the compiler's sanitizers (CPU only; no GPU, no product code).

1. AddressSanitizer + UndefinedBehaviorSanitizer: oracle/lemo_oracle.c is compiled together with
   tests/oracle_sanitize_driver.c into one instrumented executable, which calls every oracle routine on edge-case
   inputs held in exactly-sized heap blocks.  Any report (out-of-bounds access, leak, overflow, misaligned access)
   makes the run fail.
2. UndefinedBehaviorSanitizer on the shared library itself: the pins of tests/test_oracle_pins.py are run, in a child
   interpreter, against a build of the oracle with -fsanitize=undefined -fno-sanitize-recover=all.

By hand:
    gcc -O1 -g -std=c11 -fopenmp -ffp-contract=off -fsanitize=address,undefined -fno-sanitize-recover=all \\
        oracle/lemo_oracle.c tests/oracle_sanitize_driver.c -lm -o /tmp/oracle_asan && /tmp/oracle_asan
"""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "lemo_oracle.c")
DRIVER = os.path.join(ROOT, "tests", "oracle_sanitize_driver.c")
COMMON = ["gcc", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-Wall", "-Wextra", "-fno-sanitize-recover=all"]


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_asan")
    subprocess.run(COMMON + ["-O1", "-fsanitize=address,undefined", SRC, DRIVER, "-lm", "-o", exe], check=True)
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, f"sanitizer run failed:\n{r.stdout}\n{r.stderr}"
    assert "oracle sanitizer driver: ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr and "LeakSanitizer" not in r.stderr, r.stderr


def test_oracle_pins_under_undefined_behaviour_sanitizer(tmp_path):
    lib = str(tmp_path / "liblemo_oracle_ubsan.so")
    subprocess.run(COMMON + ["-O2", "-fPIC", "-shared", "-fsanitize=undefined", SRC, "-lm", "-o", lib], check=True)
    env = dict(os.environ, LEMO_ORACLE_LIB=lib, OMP_NUM_THREADS="4")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q", "-p", "no:cacheprovider"],
                       capture_output=True, text=True, env=env, cwd=ROOT, timeout=1200)
    assert r.returncode == 0, f"pins failed against the UBSan build:\n{r.stdout[-3000:]}\n{r.stderr[-3000:]}"
    assert "runtime error" not in r.stderr and "runtime error" not in r.stdout

"""The oracle under the compiler's sanitizers (CPU only).

  - address + undefined-behaviour sanitizers: oracle/sanitize_driver.c calls every function of
    oracle/potq_oracle.c on heap blocks of exactly the size it may touch;
  - undefined-behaviour sanitizer: the oracle's own pins (tests/test_oracle_*.py) run once more, in a
    child process, against a sanitized build of the shared library (POTQ_ORACLE_SANITIZE=1).
Any finding aborts the child (-fno-sanitize-recover) and fails the test.
"""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE = os.path.join(ROOT, "oracle")


def test_every_oracle_function_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize_driver")
    subprocess.run(["gcc", "-O1", "-g", "-ffp-contract=off", "-fopenmp", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-static-libasan", "-Wall", "-Wextra",
                    os.path.join(ORACLE, "potq_oracle.c"), os.path.join(ORACLE, "sanitize_driver.c"),
                    "-o", exe, "-lm"], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="2")
    env.pop("LD_PRELOAD", None)
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "oracle sanitizer driver: ok" in r.stdout


def test_oracle_pins_under_ubsan():
    env = dict(os.environ, POTQ_ORACLE_SANITIZE="1", UBSAN_OPTIONS="print_stacktrace=1")
    pins = sorted(f for f in os.listdir(os.path.join(ROOT, "tests"))
                  if f.startswith("test_oracle_") and f != "test_oracle_sanitizers.py")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        *[os.path.join("tests", f) for f in pins]], cwd=ROOT, env=env, capture_output=True,
                       text=True, timeout=900)
    assert r.returncode == 0, r.stdout[-4000:] + r.stderr[-2000:]
    assert os.path.exists(os.path.join(ORACLE, "libpotq_oracle_ubsan.so"))

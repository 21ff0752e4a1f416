"""The host code under AddressSanitizer and UndefinedBehaviorSanitizer: the library's planner,
argument checks and scheduler host code and the C oracle are built with
-fsanitize=address,undefined (tests/sanitize/build.py; the kernel launchers are stubs) and the CPU
tests of the planner, the ABI and the oracle run against that build in a child process.  Any report
of either sanitizer ends that process with an error."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TESTS = ["tests/test_planner_parity.py", "tests/test_abi.py", "tests/test_oracle_numeric.py", "tests/test_oracle_planner.py"]


def test_cpu_suites_pass_under_asan_and_ubsan():
    if os.environ.get("HZP_LIBRARY"):
        pytest.skip("already inside the sanitizer run")
    sys.path.insert(0, os.path.join(ROOT, "tests", "sanitize"))
    try:
        import build as san_build
        lib, ora = san_build.build()
    finally:
        sys.path.pop(0)
    runtime = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True, text=True).stdout.strip()
    env = dict(os.environ, HZP_LIBRARY=lib, HZP_ORACLE_LIBRARY=ora,
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=1:verify_asan_link_order=0",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1",
               LD_PRELOAD=":".join(x for x in (runtime, os.environ.get("LD_PRELOAD", "")) if x))
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + TESTS,
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert "passed" in res.stdout and "AddressSanitizer" not in tail and "runtime error" not in tail, tail

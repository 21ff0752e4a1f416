"""The library driven from a C++ program with the HIP runtime alone (no Python, no PyTorch in that
process) and checked against the C oracle: tests/native/selftest.cpp, built by tests/native/build.py."""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
EXE = os.path.join(HERE, "native", "selftest")


@pytest.mark.gpu
def test_native_selftest():
    assert os.path.exists(EXE), "run __graft_entry__.build() (or tests/native/build.py) first"
    print("native self-test", flush=True)
    res = subprocess.run([EXE], capture_output=True, text=True, timeout=100)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "selftest ok" in res.stdout


def test_native_selftest_is_built_and_reports_a_missing_gpu_cleanly():
    """Without a GPU the program must say so and leave with a status, not crash."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present: covered by the GPU test")
    assert os.path.exists(EXE), "run __graft_entry__.build() (or tests/native/build.py) first"
    res = subprocess.run([EXE], capture_output=True, text=True, timeout=100)
    assert res.returncode in (2, 3) and "selftest:" in res.stdout

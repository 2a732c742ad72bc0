"""The exchange driven from a plain C program through the C ABI (no Python binding, no torch), checked against
the oracle inside that program (tests/abi_gpu_driver.c)."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DRIVER = os.path.join(ROOT, "tests", "_build", "abi_gpu_driver")


@pytest.mark.gpu
def test_exchange_from_plain_c_matches_the_oracle():
    if not os.path.exists(DRIVER):
        pytest.skip("tests/_build/abi_gpu_driver is not built: run __graft_entry__.build() first")
    print("running", DRIVER, flush=True)
    run = subprocess.run([DRIVER], capture_output=True, text=True, timeout=100)
    assert run.returncode == 0, run.stdout + run.stderr
    assert run.stdout.strip().endswith("ok"), run.stdout
    assert run.stdout.count("identical to the oracle") == 3 + 1 + 2 + 3 + 1

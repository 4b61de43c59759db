"""The C ABI used from C++ with no Python in between (tests/host/c_abi_stress.cpp)."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))
EXE = os.path.join(HERE, "host", "c_abi_stress")


def test_native_consumer_of_the_c_abi():
    """Open job with merges and weight changes from three threads, closed jobs, the store; the program
    compares the whole pool with a host image after every round and aborts on any difference."""
    if not os.path.exists(EXE):
        pytest.skip("tests/host/c_abi_stress is not built: run python __graft_entry__.py")
    print("running", EXE, flush=True)
    run = subprocess.run([EXE, "5"], capture_output=True, text=True, timeout=110)
    print(run.stderr[-1500:], flush=True)
    assert run.returncode == 0, run.stderr[-3000:]
    assert "c_abi_stress done" in run.stdout

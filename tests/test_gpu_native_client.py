"""The C ABI driven by a program that has neither Python nor PyTorch in it (tests/native/abi_client.cpp, built by
paper_2411_07762_amd.build next to libaser.so): plain HIP allocations and streams, the five stage calls and
aser_calibrate_layers, host-side checks of Eq. 12 and of the outlier set in double precision."""
import os
import subprocess

import pytest

import paper_2411_07762_amd as aser

pytestmark = pytest.mark.gpu

CLIENT = os.path.join(os.path.dirname(aser.LIB_PATH), "aser_abi_client")


def test_native_client_runs_the_path_and_its_checks_pass():
    if not os.path.exists(CLIENT):
        pytest.skip("aser_abi_client is not built (python -m paper_2411_07762_amd.build builds it next to libaser.so)")
    res = subprocess.run([CLIENT], capture_output=True, text=True, timeout=120)
    print(res.stdout, res.stderr)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "abi_client ok" in res.stdout

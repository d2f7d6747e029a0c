"""The C ABI used from plain C++ (HIP runtime + artopk.h only, no Python in the process):
tests/abi_client/abi_client.cpp runs two round-robin steps and checks every output bit for bit
against a host computation of its own (a sort by magnitude bits and index, float32 adds in
worker order).  The binary is built together with the library."""

import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

BIN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "abi_client", "abi_client")


@pytest.mark.parametrize("args", [
    ["200003", "3"],                                        # histogram route, ragged length
    ["1", "1", "1"],                                        # the smallest problem there is
    ["300000", "4", "30000"],                               # one in ten kept
    ["262147", "2", "300", "1", "1"],                       # guess route (switched on through artopk_set_option)
    ["400001", "3", "4000", "7"],                           # seven segments, selection per segment
])
def test_abi_client(args):
    if not os.path.exists(BIN):
        pytest.skip("tests/abi_client/abi_client is not built (python -m paper_2312_02493_amd.build builds it)")
    run = subprocess.run([BIN, *args], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "abi_client: ok" in run.stdout

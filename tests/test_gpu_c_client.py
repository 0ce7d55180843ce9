"""The C ABI used from a plain C++ program (no Python binding, no PyTorch): examples/c_abi_client.cpp
allocates with hipMalloc, calls the entry points, reads back with hipMemcpy and checks every byte."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_c_client_runs_and_checks_itself():
    exe = os.path.join(ROOT, "examples", "c_abi_client")
    assert os.path.exists(exe), "build first: python -c 'import __graft_entry__ as g; g.build()'"
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and r.stdout.strip().endswith("c_abi_client ok"), (r.returncode, r.stdout[-2000:], r.stderr[-2000:])

"""The library used without the Python binding and without PyTorch: examples/c_abi_client.cpp calls the C
ABI from a plain C++ program (hipMalloc, the entry points, hipMemcpy back, every byte checked), and
examples/device_api_ring.hip runs a kernel of its own on the device API (put with SignalAdd, waitSignal,
putValue, barrier) and checks what arrived."""
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


def test_kernel_written_outside_the_library_on_the_device_api():
    exe = os.path.join(ROOT, "examples", "device_api_ring")
    assert os.path.exists(exe), "build first: python -c 'import __graft_entry__ as g; g.build()'"
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and r.stdout.strip().endswith("device_api_ring ok"), (r.returncode, r.stdout[-2000:], r.stderr[-2000:])

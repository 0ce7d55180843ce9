"""Builds libmi_shmem.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libmi_shmem.so")
ROOT = os.path.dirname(HERE)
CEILINGS_PATH = os.path.join(ROOT, "bench_ceilings")
CLIENT_PATH = os.path.join(ROOT, "examples", "c_abi_client")


def hipcc() -> str:
    return shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def build(verbose: bool = False) -> str:
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-pthread",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-command-line-argument",
           os.path.join(CSRC, "mi_shmem.hip"), "-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    # measurement aid: plain read / write / copy ceilings of the box (bench.py --ceilings)
    cmd2 = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-I", ROOT,
            os.path.join(ROOT, "bench_ceilings.hip"), "-o", CEILINGS_PATH]
    if verbose:
        print(" ".join(cmd2), flush=True)
    subprocess.run(cmd2, check=True)
    # a client of the C ABI without Python (host code only; tests/test_gpu_c_client.py runs it)
    cmd3 = [hipcc(), "-O2", "-std=c++17", "-Wall", "-I", os.path.join(ROOT, "include"),
            os.path.join(ROOT, "examples", "c_abi_client.cpp"), "-o", CLIENT_PATH,
            "-L", HERE, "-lmi_shmem", "-Wl,-rpath,$ORIGIN/../paper_2511_15076_amd"]
    if verbose:
        print(" ".join(cmd3), flush=True)
    subprocess.run(cmd3, check=True)
    # a kernel written outside the library on the device API of include/mi_shmem_device.hpp
    cmd4 = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wno-unused-command-line-argument", "-I", os.path.join(ROOT, "include"),
            os.path.join(ROOT, "examples", "device_api_ring.hip"), "-o", os.path.join(ROOT, "examples", "device_api_ring"),
            "-L", HERE, "-lmi_shmem", "-Wl,-rpath,$ORIGIN/../paper_2511_15076_amd"]
    if verbose:
        print(" ".join(cmd4), flush=True)
    subprocess.run(cmd4, check=True)
    return LIB_PATH


if __name__ == "__main__":
    build(True)

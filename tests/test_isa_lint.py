"""Assembly lint (CPU only): no store or atomic in the compiled device code may name a data register
that overlaps its own address register.  hipcc once allocated the address pair of a vector store inside
the tuple that held the vector to be stored (wrong bytes, no fault); the parity tests caught it, this
check catches the pattern at build time, in every kernel and on every path, tested or not."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2511_15076_amd", "csrc", "mi_shmem.hip")


def regs(op):
    """'v[20:23]' -> {20,21,22,23}; 'v7' -> {7}; anything else -> empty."""
    m = re.fullmatch(r"v\[(\d+):(\d+)\]", op)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.fullmatch(r"v(\d+)", op)
    return {int(m.group(1))} if m else set()


def overlapping(asm_text):
    bad = []
    for n, line in enumerate(asm_text.splitlines(), 1):
        line = line.split(";")[0].strip()
        m = re.match(r"(global_store_\w+|global_atomic_\w+|flat_store_\w+|flat_atomic_\w+)\s+(.*)", line)
        if not m:
            continue
        ops = [o.strip() for o in m.group(2).split(",")]
        vec = [o for o in ops if o.startswith("v")]
        if m.group(1).startswith(("global_atomic", "flat_atomic")) and len(vec) == 3:
            vec = vec[1:]                      # returning atomic: destination, address, data
        # only the form with a 64-bit address pair ("off"): with a scalar base the 32-bit offset register may
        # legitimately be a zero that the data tuple shares (e.g. the high half of a compare value of 0)
        if not any(o.split()[0] == "off" for o in ops if o) or len(vec) < 2 or len(regs(vec[0])) != 2:
            continue
        if regs(vec[0]) & regs(vec[1]):
            bad.append((n, line))
    return bad


def test_lint_recognises_the_pattern():
    assert overlapping("\tglobal_store_dwordx4 v[22:23], v[20:23], off offset:1024 nt\n")
    assert overlapping("\tglobal_atomic_or_x2 v[4:5], v[2:3], v[3:4], off sc0\n")
    assert not overlapping("\tglobal_atomic_cmpswap_x2 v[2:3], v17, v[14:17], s[62:63] sc0\n")   # shared zero
    assert not overlapping("\tglobal_store_dwordx4 v[22:23], v[28:31], off nt\n"
                           "\tglobal_store_dwordx4 v8, v[0:3], s[4:5]\n"
                           "\tglobal_atomic_or_x2 v[44:45], v[38:39], v[40:41], off sc0\n"
                           "\tglobal_load_dwordx4 v[0:3], v[0:1], off\n")


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="no hipcc")
def test_no_store_overlaps_its_address(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    out = tmp_path / "mi_shmem.s"
    subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                    "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-S", "--cuda-device-only", SRC,
                    "-o", str(out)], check=True, capture_output=True)
    bad = overlapping(out.read_text())
    assert not bad, bad[:5]

"""The library's HIP-free host logic (allocator, descriptor validation) compiled for the CPU and held
against the oracle: same allocation policy offset by offset, same verdict on every descriptor."""
import os
import subprocess

import numpy as np
import pytest

import oracle
import workgen

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def harness(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("hostlogic") / "host_logic_harness")
    subprocess.run(["g++", "-O1", "-std=c++17", "-Wall", "-Werror", "-o", exe, os.path.join(HERE, "host_logic_harness.cpp")],
                   check=True)

    def run(lines):
        out = subprocess.run([exe], input="\n".join(lines) + "\n", capture_output=True, text=True, check=True)
        return out.stdout.split("\n")[:-1]
    return run


def test_allocator_follows_the_oracle_policy(harness):
    seg = 1 << 16
    rng = np.random.default_rng(5)
    w = oracle.World(1, seg, oracle.EAGER, 0)
    cmds, want, live = ["I 0 %d" % seg], ["0"], []
    for step in range(3000):
        r = rng.random()
        if live and r < 0.45:
            off = live.pop(int(rng.integers(0, len(live))))
            assert w.free(off) == 0
            cmds.append(f"F {off}"); want.append("1")
        elif r < 0.5:
            bogus = int(rng.integers(0, seg // 256)) * 256 + 128          # never a block start
            assert w.free(bogus) != 0
            cmds.append(f"F {bogus}"); want.append("0")
        elif r < 0.8:
            n = int(rng.integers(1, 3000))
            off = w.malloc(n)
            cmds.append(f"A 256 {n}"); want.append(str(off))
            if off >= 0:
                live.append(off)
        else:
            al = 1 << int(rng.integers(0, 13))
            n = int(rng.integers(1, 3000))
            off = w.align(al, n)
            cmds.append(f"A {al} {n}"); want.append(str(off))
            if off >= 0:
                assert off % max(al, 256) == 0
                live.append(off)
    cmds.append("N"); want.append(None)
    got = harness(cmds)
    assert got[:-1] == want[:-1]
    assert int(got[-1].split()[0]) == len(live) == w.live_blocks()
    assert "-1" in want and any(x not in ("0", "1", "-1") for x in want)     # the run filled the heap and allocated


def test_allocator_edge_cases(harness):
    out = harness(["I 0 4096", "A 256 0", "A 3 8", "A 0 8", "A 8192 8", "A 256 4097", "A 256 4096", "A 256 1", "F 0", "F 0",
                   "A 1 1", "A 1 1", "N",
                   # a heap whose device address is only 256-aligned: 1024-aligned blocks sit at odd offsets
                   "I 768 4096", "A 1024 10", "A 1024 10"])
    assert out == ["0", "-1", "-1", "-1", "-1", "-1", "0", "-1", "1", "0", "0", "256", "2 1", "0", "256", "1280"]


def test_descriptor_validation_agrees_with_the_oracle(harness):
    npes, seg = 3, 1 << 12
    rng = np.random.default_rng(17)
    edge = [0, 1, 2, 3, 4, 7, 8, 9, 255, 256, seg // 2, seg - 9, seg - 8, seg - 7, seg - 1, seg, seg + 1, seg + 8,
            2**32, 2**63 - 1, 2**63, 2**64 - 8, 2**64 - 1]
    strides = [-2**63, -1, 0, 1, 2, 3, 17, seg // 8, seg, seg + 1, 2**31, 2**62, 2**63 - 1]
    ops = np.zeros(6000, dtype=workgen.OP_DESC)
    pick = lambda seq: seq[int(rng.integers(len(seq)))]
    mostly = lambda sane, odd: pick(sane) if rng.random() < 0.85 else pick(odd)     # one odd field is enough to reject
    for d in ops:
        d["kind"] = np.uint32(mostly([0, 1, 2, 3], [4, 2**32 - 1]))
        d["pe_self"] = np.uint32(mostly([0, 1, 2], [3, 2**31]))
        d["pe"] = np.uint32(mostly([0, 1, 2], [3, 2**32 - 1]))
        d["elem_bytes"] = np.uint32(mostly([1, 2, 4, 8], [0, 3, 16]))
        d["local_off"] = np.uint64(mostly([0, 8, 64, 256, seg // 2, seg - 8, seg], edge))
        d["sym_off"] = np.uint64(mostly([0, 16, 128, seg // 4, seg - 16, seg], edge))
        d["count"] = np.uint64(mostly([0, 1, 2, 5, 8, 100, seg // 8, seg // 2], edge))
        d["local_stride"] = np.int64(mostly([1, 1, 2, 3, seg // 8], strides))
        d["sym_stride"] = np.int64(mostly([1, 1, 2, 17], strides))
    names = ops.dtype.names
    assert names[:9] == ("kind", "pe_self", "pe", "elem_bytes", "local_off", "sym_off", "count", "local_stride", "sym_stride")
    cmds = [f"V {npes} {seg} " + " ".join(str(int(d[n])) for n in names[:9]) for d in ops]
    got = harness(cmds)
    w = oracle.World(npes, seg, oracle.EAGER, 0)
    want = ["1" if w.op_batch(ops[i:i + 1], 0) == 0 else "0" for i in range(len(ops))]
    assert got == want
    assert 300 < want.count("1") < len(want) - 300          # both verdicts are well represented


def test_single_op_argument_checks_report_what_the_oracle_reports(harness):
    # put / get, iput / iget and the atomics over edge values of every argument: same status code as the
    # oracle, in particular the same one when several arguments are wrong at once.  The local side is kept
    # valid (the library takes any device pointer there and checks only its alignment).
    npes, seg = 3, 1 << 12
    rng = np.random.default_rng(23)
    pick = lambda seq: seq[int(rng.integers(len(seq)))]
    mostly = lambda sane, odd: pick(sane) if rng.random() < 0.8 else pick(odd)
    offs = [0, 1, 2, 4, 8, 9, 64, seg // 2, seg - 16, seg - 8, seg - 4, seg - 1, seg]
    odd_offs = [seg + 1, seg + 8, 2**32, 2**63, 2**64 - 8, 2**64 - 1]
    counts = [0, 1, 2, 3, 8, 100, seg // 8, seg // 2, seg - 1, seg]
    odd_counts = [seg + 1, 2**32, 2**63, 2**64 - 1]
    strides = [1, 1, 2, 3, 17, seg // 8, seg]
    odd_strides = [0, -1, -2**63, seg + 1, 2**40, 2**63 - 1]
    pes, odd_pes = [0, 1, 2], [-1, 3, 2**31 - 1, -2**31]
    w = oracle.World(npes, seg, oracle.EAGER, 0)
    cmds, want = [], []
    for _ in range(4000):
        me, pe = mostly(pes, odd_pes), mostly(pes, odd_pes)
        so = mostly(offs, odd_offs)
        kind = int(rng.integers(0, 5))
        if kind < 2:                                    # put / get of n bytes; local range valid
            n = mostly(counts, odd_counts)
            lo = 0
            cmds.append(f"C {npes} {seg} {me} {pe} {so} {n}")
            if n > seg:                                 # the oracle also checks the local range: keep that out of the verdict
                rc = -5 if (0 <= me < npes and 0 <= pe < npes) else -4      # out of range / invalid PE
            else:
                rc = w.put(me, so, lo, n, pe) if kind == 0 else w.get(me, lo, so, n, pe)
            want.append(str(rc))
        elif kind < 4:                                  # iput / iget; local side: offset 0 or 4, stride 1, fits whenever the count does
            eb = mostly([1, 2, 4, 8], [0, 3, 16])
            ss = mostly(strides, odd_strides)
            n = mostly([0, 1, 2, 5, 60, seg // 8], odd_counts)
            lo = pick([0, 4, 8])
            cmds.append(f"S {npes} {seg} {me} {pe} {so} {ss} {lo} 1 {n} {eb}")
            if eb in (1, 2, 4, 8) and n * eb + lo > seg:
                cmds.pop()                              # the local span would not fit the oracle's heap: not a case
                continue
            rc = w.iput(me, so, lo, ss, 1, n, eb, pe) if kind == 2 else w.iget(me, lo, so, 1, ss, n, eb, pe)
            want.append(str(rc))
        else:
            cmds.append(f"M {npes} {seg} {me} {pe} {so}")
            want.append(str(w.signal_add(me, so, 1, pe)))     # a remote fetch-add: the atomics' argument checks
    got = harness(cmds)
    assert got == want
    assert {"0", "-3", "-4", "-5", "-6"} <= set(want)   # every class of verdict occurred

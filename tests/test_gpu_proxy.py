"""GPU tests of the proxy-style executor: descriptors enqueued by GPU threads into a ring in
pinned host memory, carried out by a host thread.  Differential against the oracle and against
the device path (shmem_op_batch) on the same seeded descriptor tables: identical heaps."""
import numpy as np
import pytest
import torch

import oracle
import workgen

pytestmark = pytest.mark.gpu

sh = pytest.importorskip("paper_2511_15076_amd")
from gpu_util import heaps_of, shmem_world, to_dev  # noqa: E402


def seeded_heaps(npes, hb, seed):
    return np.stack([workgen.random_words(seed + p, hb // 8).view(np.uint8) for p in range(npes)])


def oracle_heaps(init, ops, every):
    npes, hb = init.shape
    w = oracle.World(npes, hb, oracle.SHUFFLED, 4)
    for p in range(npes):
        w.heap(p)[:] = init[p]
    assert w.op_batch(ops, every) == 0
    out = w.heaps().copy()
    w.close()
    return out


@pytest.mark.parametrize("entries,wgs", [(64, 1), (1024, 4), (1 << 14, 16)])
def test_proxy_matches_oracle_and_device_path(entries, wgs):
    # the config-1 table: 10,000 random puts/gets of 8 B..4 KiB on 4 PEs, conflict-free within windows of
    # 100; the proxy runs them strictly in table order, which is one of the orders the windows allow
    npes, hb = 4, 1 << 20
    ops = workgen.cfg1_op_table()
    init = seeded_heaps(npes, hb, 900)
    want = oracle_heaps(init, ops, 100)
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        d_ops = to_dev(ops)
        px = sh.proxy_create(entries)                      # 64 entries: the ring wraps 156 times
        sh.proxy_submit(px, d_ops, len(ops), wgs)
        sh.proxy_quiet(px)
        st = sh.proxy_stats(px)
        assert st == {"submitted": len(ops), "executed": len(ops), "rejected": 0}
        got_proxy = heaps_of(heap, npes)
        sh.proxy_destroy(px)
        assert np.array_equal(got_proxy, want)
        heap.copy_(torch.from_numpy(init.reshape(-1)))    # the device path on the same table
        sh.op_batch(d_ops, len(ops), 100, 2)
        sh.stream_sync()
        assert np.array_equal(heaps_of(heap, npes), got_proxy)


@pytest.mark.parametrize("entries,nops,wgs", [(2, 700, 1), (4, 900, 2), (8, 1000, 1), (32, 3000, 3)])
def test_proxy_ring_shorter_than_a_wavefront(entries, nops, wgs):
    # one submission of far more descriptors than the ring holds, and a ring shorter than the 64 lanes of a
    # wave: the higher lanes' slots only come free after the host has taken out what the lower lanes of the
    # SAME wave publish, so no lane may spin on its slot while the others wait for it
    npes, hb = 4, 1 << 18
    ops = workgen.cfg1_op_table(seed=4242 + entries, npes=npes, heap_bytes=hb, nops=nops)
    init = seeded_heaps(npes, hb, 300 + entries)
    want = oracle_heaps(init, ops, 100)
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        px = sh.proxy_create(entries)
        sh.proxy_submit(px, to_dev(ops), len(ops), wgs)
        sh.proxy_quiet(px)
        assert sh.proxy_stats(px) == {"submitted": nops, "executed": nops, "rejected": 0}
        assert np.array_equal(heaps_of(heap, npes), want)
        sh.proxy_destroy(px)
        sh.stream_sync()                                   # no producer gave up


def test_proxy_strided_and_several_submissions():
    npes, hb = 3, 1 << 16
    init = seeded_heaps(npes, hb, 50)
    ops = np.zeros(6, dtype=workgen.OP_DESC)
    def op(i, kind, me, pe, eb, lo, so, cnt, ls=1, ss=1):
        ops[i] = (kind, me, pe, eb, lo, so, cnt, ls, ss, 0)
    op(0, workgen.OP_IPUT, 0, 1, 4, 0, 4096, 100, 3, 5)       # strided both sides
    op(1, workgen.OP_IGET, 2, 0, 8, 8192, 1024, 33, 2, 7)
    op(2, workgen.OP_PUT, 1, 2, 1, 4096, 20000, 777)           # reads what op 0 wrote: order matters
    op(3, workgen.OP_GET, 0, 2, 1, 30000, 20000, 777)          # reads what op 2 wrote
    op(4, workgen.OP_IPUT, 1, 1, 2, 40000, 50000, 0, 1, 1)     # empty
    op(5, workgen.OP_PUT, 2, 2, 1, 100, 60000, 13)             # to itself
    want = oracle_heaps(init, ops, 1)                          # quiet + barrier after every op = in order
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        d_ops = to_dev(ops)
        px = sh.proxy_create(2)                                # the smallest ring
        for i in range(0, 6, 2):                               # three submissions of two descriptors
            sh.proxy_submit(px, d_ops.data_ptr() + 64 * i, 2, 1)
        sh.proxy_quiet(px)
        assert sh.proxy_stats(px)["executed"] == 6
        assert np.array_equal(heaps_of(heap, npes), want)
        sh.proxy_destroy(px)


def test_proxy_rejects_bad_descriptors_on_the_host():
    npes, hb = 2, 1 << 16
    init = seeded_heaps(npes, hb, 60)
    ops = np.zeros(4, dtype=workgen.OP_DESC)
    ops[0] = (workgen.OP_PUT, 0, 1, 1, 0, 1024, 64, 1, 1, 0)
    ops[1] = (workgen.OP_PUT, 0, 5, 1, 0, 2048, 64, 1, 1, 0)          # no such PE
    ops[2] = (workgen.OP_GET, 1, 0, 1, 0, hb - 8, 64, 1, 1, 0)        # runs past the segment
    ops[3] = (workgen.OP_PUT, 1, 0, 1, 128, 4096, 32, 1, 1, 0)
    want = init.copy()
    want[1, 1024:1088] = init[0, 0:64]
    want[0, 4096:4128] = init[1, 128:160]
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        px = sh.proxy_create(16)
        sh.proxy_submit(px, to_dev(ops), 4, 1)
        with pytest.raises(sh.ShmemError) as ei:
            sh.proxy_quiet(px)
        assert ei.value.status == sh.ERR_DEVICE_FAULT and ei.value.first_bad_index == 1
        assert sh.proxy_stats(px) == {"submitted": 4, "executed": 4, "rejected": 2}
        assert np.array_equal(heaps_of(heap, npes), want)           # the valid ones were still carried out
        sh.proxy_destroy(px)


def test_proxy_argument_checks():
    with shmem_world(2, 1 << 16):
        for bad in (0, 1, 3, 100, 1 << 21):
            with pytest.raises(sh.ShmemError) as ei:
                sh.proxy_create(bad)
            assert ei.value.status == sh.ERR_INVALID_ARG
        px = sh.proxy_create(8)
        t = torch.zeros(256, dtype=torch.uint8, device="cuda:0")
        with pytest.raises(sh.ShmemError):
            sh.proxy_submit(px, t, 1, 0)
        with pytest.raises(sh.ShmemError):
            sh.proxy_submit(px, t.data_ptr() + 8, 1, 1)            # misaligned table
        sh.proxy_submit(px, t, 0, 1)                               # nothing to do
        sh.proxy_quiet(px)
        sh.proxy_destroy(px)
        with pytest.raises(sh.ShmemError):
            sh.proxy_destroy(px)                                   # not a live proxy any more
        sh.proxy_create(8)                                         # left alive: finalize stops its thread

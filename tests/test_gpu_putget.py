"""GPU parity, bit-exact: put / get / iput / iget, the descriptor-table
executor (configuration 1 at full size) and the bandwidth-sweep cell
(configuration 2's op shapes at sizes that span several chunks and a ragged
tail), against the CPU oracle on the same seeded inputs."""
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


def oracle_world(init, seed=3):
    npes, hb = init.shape
    w = oracle.World(npes, hb, oracle.SHUFFLED, seed)
    for p in range(npes):
        w.heap(p)[:] = init[p]
    return w


@pytest.mark.parametrize("wgs", [1, 2, 3, 8])       # 1, 2 and 8 are the team sizes bench.py times
def test_config1_full_table(wgs):
    npes, hb = 4, 1 << 20
    ops = workgen.cfg1_op_table()                       # 10,000 ops, batches of 100
    init = seeded_heaps(npes, hb, workgen.BASE_SEED + 100)
    w = oracle_world(init)
    assert w.op_batch(ops, 100) == 0
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        dops = to_dev(ops)
        sh.op_batch(dops, len(ops), 100, wgs)
        sh.stream_sync()
        got = heaps_of(heap, npes)
    assert np.array_equal(got, w.heaps())


@pytest.mark.parametrize("batch,nops,wgs", [(1, 70, 2), (7, 203, 1), (64, 640, 3), (65, 650, 2), (129, 1000, 4),
                                            (1000, 1000, 2), (0, 300, 2)])
def test_table_window_sizes(batch, nops, wgs):
    # windows shorter than, equal to and longer than the 64 descriptors a wave reads at a time, a last
    # window that is not full, and a single window (quiet_every = 0): the executor prefetches the next
    # batch of descriptors across window ends, so every boundary shape is exercised
    npes, hb = 4, 1 << 18
    gen_batch = batch if batch else nops
    ops = workgen.cfg1_op_table(seed=workgen.BASE_SEED + 7 + batch, npes=npes, heap_bytes=hb, nops=nops,
                                batch=gen_batch, max_log2=10)
    init = seeded_heaps(npes, hb, 31 + batch)
    w = oracle_world(init)
    assert w.op_batch(ops, batch) == 0
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        sh.op_batch(to_dev(ops), len(ops), batch, wgs)
        sh.stream_sync()
        got = heaps_of(heap, npes)
    assert np.array_equal(got, w.heaps())


def test_table_with_strided_and_large_ops_and_device_fault():
    npes, hb = 3, 1 << 20
    init = seeded_heaps(npes, hb, 555)
    ops = np.zeros(9, dtype=workgen.OP_DESC)
    # disjoint regions by construction
    ops[7] = (workgen.OP_IGET, 1, 0, 8, 1040000, 1040008, 1, 2**31, 2**62, 0)   # one element: any stride is in range
    ops[8] = (workgen.OP_IPUT, 2, 1, 4, 1041000, 1041004, 0, 2**40, 1, 0)       # no element at all
    ops[0] = (workgen.OP_PUT, 0, 1, 1, 0, 0, 200000, 1, 1, 0)            # large: whole team
    ops[1] = (workgen.OP_IPUT, 1, 2, 4, 300000, 300000, 5000, 3, 5, 0)   # local stride 3, remote 5
    ops[2] = (workgen.OP_IGET, 2, 0, 8, 500000, 600000, 700, 2, 7, 0)
    ops[3] = (workgen.OP_GET, 0, 2, 1, 800003, 900001, 1237, 1, 1, 0)    # byte-granular, odd alignment
    ops[4] = (workgen.OP_PUT, 1, 1, 1, 8, 950000, 0, 1, 1, 0)            # zero bytes
    ops[5] = (workgen.OP_PUT, 2, 7, 1, 0, 0, 8, 1, 1, 0)                 # bad remote PE -> rejected
    ops[6] = (workgen.OP_IPUT, 0, 1, 2, 1000000, 1000000, 100, 9, 1, 0)
    w = oracle_world(init)
    assert w.op_batch(ops, 0) == -4                     # the oracle rejects op 5 too, the rest is done
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        sh.op_batch(to_dev(ops), len(ops), 0, 2)
        with pytest.raises(sh.ShmemError) as e:
            sh.stream_sync()
        assert e.value.status == sh.ERR_DEVICE_FAULT and e.value.first_bad_index == 5
        sh.stream_sync()                                # the fault word was cleared
        got = heaps_of(heap, npes)
    assert np.array_equal(got, w.heaps())


@pytest.mark.parametrize("wgs", [1, 5, 16, 33])
def test_table_large_ops_take_the_streaming_copy(wgs):
    # ops above 64 KiB are done by the whole team; in teams of 16 workgroups and more those with 16-byte
    # aligned ends go through the pipelined loop (whole 4 KiB tasks + a tail), everything else through
    # the generic copy -- team sizes and op sizes on both sides of each rule
    npes, hb = 4, 8 << 20
    init = seeded_heaps(npes, hb, 808)
    M = 1 << 20
    ops = np.zeros(6, dtype=workgen.OP_DESC)
    ops[0] = (workgen.OP_PUT, 0, 1, 1, 0, 4 * M, 65536 + 16, 1, 1, 0)
    ops[1] = (workgen.OP_GET, 1, 2, 1, 16, 5 * M + 256, M + 4096 + 48, 1, 1, 0)
    ops[2] = (workgen.OP_PUT, 2, 3, 1, 8, 6 * M + 8, 300000, 1, 1, 0)          # 8-byte aligned only: generic copy
    ops[3] = (workgen.OP_GET, 3, 0, 1, 2 * M, 7 * M, 4096 * 37, 1, 1, 0)       # whole tasks, no tail
    ops[4] = (workgen.OP_PUT, 1, 1, 1, 2 * M, 6 * M, 70000, 1, 1, 0)           # to itself
    ops[5] = (workgen.OP_PUT, 3, 2, 1, 4 * M, 2 * M + 4096, 4096 * 16 + 4080, 1, 1, 0)
    w = oracle_world(init)
    assert w.op_batch(ops, 0) == 0
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        sh.op_batch(to_dev(ops), len(ops), 0, wgs)
        sh.stream_sync()
        got = heaps_of(heap, npes)
    assert np.array_equal(got, w.heaps())


@pytest.mark.parametrize("seed", [1, 2, 3, 4, 5, 6])
def test_random_mixed_tables_match_oracle(seed):
    # Random tables of all four kinds with random element sizes, strides, counts (zero included) and byte
    # alignments, executed by the table executor AND by the proxy executor.  Inside a window every op owns
    # one local and one remote 4 KiB stripe, so the table is race-free by construction; later windows
    # reuse stripes, so an op that is dropped, duplicated or misplaced shows in the whole-heap comparison.
    rng = np.random.default_rng(1000 + seed)
    npes = int(rng.integers(2, 6))
    stripes, sb = 48, 4096
    hb = 2 * stripes * sb
    window = int(rng.integers(5, stripes // 2))
    nwin = 12
    ops = np.zeros(window * nwin, dtype=workgen.OP_DESC)
    for wdx in range(nwin):
        # per PE, which local / remote stripes are still free in this window
        free_l = [list(rng.permutation(stripes)) for _ in range(npes)]
        free_r = [list(rng.permutation(stripes)) for _ in range(npes)]
        for k in range(window):
            me, pe = int(rng.integers(0, npes)), int(rng.integers(0, npes))
            lo = int(free_l[me].pop()) * sb                       # local stripes: first half of the heap
            so = (stripes + int(free_r[pe].pop())) * sb           # remote stripes: second half
            kind = int(rng.integers(0, 4))
            if kind < 2:
                n = int(rng.choice([0, 1, 2, 7, 8, 9, 16, 31, 64, 100, 255, 256, 1000, 2048, 3000, sb - 64]))
                a, b = int(rng.integers(0, 64)), int(rng.integers(0, 64))
                ops[wdx * window + k] = (kind, me, pe, 1, lo + a, so + b, n, 1, 1, 0)
            else:
                eb = int(rng.choice([1, 2, 4, 8]))
                ls, ss = int(rng.integers(1, 10)), int(rng.integers(1, 10))
                room = sb // eb
                cnt = int(rng.integers(0, (room - 8) // max(ls, ss) + 1))
                a, b = int(rng.integers(0, 4)) * eb, int(rng.integers(0, 4)) * eb
                ops[wdx * window + k] = (kind, me, pe, eb, lo + a, so + b, cnt, ls, ss, 0)
    init = seeded_heaps(npes, hb, 300 + seed)
    w = oracle_world(init)
    assert w.op_batch(ops, window) == 0
    want = w.heaps()
    wgs = int(rng.choice([1, 2, 3, 8, 16, 33]))          # from 16 on the executor is the variant with the streaming copy
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        sh.op_batch(to_dev(ops), len(ops), window, wgs)
        sh.stream_sync()
        assert np.array_equal(heaps_of(heap, npes), want), "table executor"
        # the proxy carries out descriptors one after the other in table order: the same result
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        px = sh.proxy_create(64)
        sh.proxy_submit(px, to_dev(ops), len(ops), 2)
        sh.proxy_quiet(px)
        assert np.array_equal(heaps_of(heap, npes), want), "proxy executor"
        sh.proxy_destroy(px)


def test_single_ops_byte_granular():
    npes, hb = 3, 1 << 18
    init = seeded_heaps(npes, hb, 42)
    w = oracle_world(init)
    rng = np.random.default_rng(1)
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        # each op works in its own 8 KiB stripe: no conflicts in either model
        for k in range(30):
            n = int(rng.choice([0, 1, 3, 7, 8, 15, 16, 17, 63, 64, 100, 255, 1024, 2049, 4000]))
            a, b = int(rng.integers(0, 96)), int(rng.integers(0, 96))
            me, pe = int(rng.integers(0, npes)), int(rng.integers(0, npes))
            lo, so = k * 8192 + a, k * 8192 + 4096 + b
            if k % 2 == 0:
                assert w.put(me, so, lo, n, pe) == 0
                sh.put(me, base + so, sh.ptr(base + lo, me), n, pe)
            else:
                assert w.get(me, lo, so, n, pe) == 0
                sh.get(me, sh.ptr(base + lo, me), base + so, n, pe)
            sh.quiet(me)
            w.quiet(me)
        sh.barrier_all()
        got = heaps_of(heap, npes)
    w.barrier_all()
    assert np.array_equal(got, w.heaps())


def test_single_large_put_get():
    # stand-alone puts / gets of 1 MiB and more: 16-byte aligned ends take the streaming kernel (whole
    # 4 KiB tasks plus a generic tail), anything else the generic copy; several sizes around the task and
    # grid boundaries, neighbouring bytes checked through the whole-heap comparison
    npes, hb = 2, 40 << 20
    init = seeded_heaps(npes, hb, 77)
    w = oracle_world(init)
    half = hb // 2
    cases = [(1 << 20, 0, 0), ((1 << 20) + 4096 + 48, 256, 512), ((5 << 20) + 8, 16, 16), ((3 << 20) + 16, 8, 16),
             ((2 << 20) + 4095, 32, 4096), (16 << 20, 0, 0), ((16 << 20) - 4096 + 16, 4096, 16)]
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        for k, (n, a, b) in enumerate(cases):
            lo, so = a, half + b
            if k % 2 == 0:
                assert w.put(0, so, lo, n, 1) == 0
                sh.put(0, base + so, sh.ptr(base + lo, 0), n, 1)
            else:
                assert w.get(1, lo, so, n, 0) == 0
                sh.get(1, sh.ptr(base + lo, 1), base + so, n, 0)
            sh.barrier_all()
            w.barrier_all()
            assert np.array_equal(heaps_of(heap, npes), w.heaps()), (k, n, a, b)


@pytest.mark.parametrize("eb", [1, 2, 4, 8])
def test_single_iput_iget(eb):
    npes, hb = 2, 1 << 20
    init = seeded_heaps(npes, hb, 77 + eb)
    w = oracle_world(init)
    rng = np.random.default_rng(eb)
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        half = hb // 2
        for k in range(12):
            ds, ss = int(rng.integers(1, 9)), int(rng.integers(1, 9))
            if k % 3 == 0:
                ds = 1
            if k % 3 == 1:
                ss = 1
            n = int(rng.integers(0, 3000))
            so = int(rng.integers(0, 8)) * eb                    # source in the low half
            do = half + int(rng.integers(0, 8)) * eb            # destination in the high half
            if k % 2 == 0:
                assert w.iput(0, do, so, ds, ss, n, eb, 1) == 0
                sh.iput(0, base + do, sh.ptr(base + so, 0), ds, ss, n, eb, 1)
            else:
                assert w.iget(1, do, so, ds, ss, n, eb, 0) == 0
                sh.iget(1, sh.ptr(base + do, 1), base + so, ds, ss, n, eb, 0)
            w.barrier_all()
            got = heaps_of(heap, npes)
            assert np.array_equal(got, w.heaps()), (k, ds, ss, n)


SWEEP_CASES = [
    # kind, count, eb, remote_stride, local_stride, ops_per_pe, nslots, wgs
    (workgen.OP_PUT, 8, 1, 1, 1, 5, 3, 1),
    (workgen.OP_GET, 64, 1, 1, 1, 7, 2, 2),
    # small messages: 8- and 16-byte vectors, group sizes from 1 to 64 lanes, op counts that leave ragged rounds
    (workgen.OP_PUT, 16, 1, 1, 1, 301, 301, 1),
    (workgen.OP_GET, 24, 1, 1, 1, 130, 130, 2),
    (workgen.OP_PUT, 48, 1, 1, 1, 77, 77, 1),
    (workgen.OP_GET, 256, 1, 1, 1, 77, 40, 1),
    (workgen.OP_PUT, 504, 1, 1, 1, 33, 33, 1),
    (workgen.OP_GET, 512, 1, 1, 1, 131, 131, 3),
    (workgen.OP_PUT, 4096, 1, 1, 1, 9, 4, 3),
    (workgen.OP_PUT, 14352, 1, 1, 1, 6, 3, 2),          # the paper's MoE dispatch message size
    (workgen.OP_GET, 14336, 1, 1, 1, 6, 3, 5),          # ... and its combine message size
    (workgen.OP_GET, 1040, 1, 1, 1, 37, 5, 3),          # one full KiB and one 16-byte vector
    (workgen.OP_PUT, 3 * 1024 + 80, 1, 1, 1, 21, 21, 2),
    (workgen.OP_PUT, (1 << 20) + 48, 1, 1, 1, 3, 3, 16),  # many chunks and a 48-byte tail
    (workgen.OP_PUT, (1 << 20) + 24, 1, 1, 1, 3, 2, 16),  # several chunks and a ragged tail
    (workgen.OP_GET, (1 << 20) + 8, 1, 1, 1, 2, 1, 7),
    (workgen.OP_IPUT, 5000, 4, 1, 2, 3, 2, 3),          # gather (local side strided)
    (workgen.OP_IPUT, 5000, 4, 64, 1, 3, 2, 4),         # scatter
    (workgen.OP_IPUT, 3001, 4, 16, 8, 2, 2, 2),         # both strided
    (workgen.OP_IGET, 5003, 4, 4, 1, 3, 2, 3),          # gather from remote
    (workgen.OP_IGET, 2000, 4, 1, 32, 2, 1, 1),
    (workgen.OP_IGET, 1500, 8, 3, 5, 2, 2, 2),
]


@pytest.mark.parametrize("case", SWEEP_CASES)
def test_copy_sweep_cell(case):
    kind, count, eb, rs, ls, nops, nslots, wgs = case
    npes = 8
    strided = kind >= workgen.OP_IPUT
    rspan = ((count - 1) * rs + 1) * eb if strided else count
    lspan = ((count - 1) * ls + 1) * eb if strided else count
    rslot = (rspan + 255) // 256 * 256
    lslot = (lspan + 255) // 256 * 256 + 256
    hb = ((rslot + lslot) * nslots + 4096 + 255) // 256 * 256
    init = seeded_heaps(npes, hb, 900 + count % 97)
    w = oracle_world(init)
    local_off, remote_off = 0, lslot * nslots + 256
    for p in range(npes):
        peer = (p + 1) % npes
        for k in range(nops):
            s = k % nslots
            lo, ro = local_off + s * lslot, remote_off + s * rslot
            if kind == workgen.OP_PUT:
                rc = w.put(p, ro, lo, count, peer)
            elif kind == workgen.OP_GET:
                rc = w.get(p, lo, ro, count, peer)
            elif kind == workgen.OP_IPUT:
                rc = w.iput(p, ro, lo, rs, ls, count, eb, peer)
            else:
                rc = w.iget(p, lo, ro, ls, rs, count, eb, peer)
            assert rc == 0
    w.barrier_all()
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        sh.copy_sweep(kind, base + remote_off, base + local_off, count, eb, rs, ls, rslot, lslot,
                      nslots, nops, wgs)
        sh.stream_sync()
        got = heaps_of(heap, npes)
    assert np.array_equal(got, w.heaps())
    assert not np.array_equal(got, init)


# Bandwidth cells: whole 4 KiB tasks, at least one workgroup per compute unit -> the streaming copy (wave-specialised
# workgroups, LDS ring, every PE's task list rotated).  Team sizes that are not powers of two, slots used several times
# over, unequal slot pitches, a PE that is its own peer, and task counts that leave some workgroups one task short.
STREAM_CASES = [
    # npes, kind, count, ops_per_pe, nslots, wgs_per_pe
    (8, workgen.OP_PUT, 4096, 600, 600, 32),
    (8, workgen.OP_GET, 8192, 300, 77, 256),
    (8, workgen.OP_PUT, 20480, 131, 131, 64),
    (3, workgen.OP_GET, 12288, 500, 500, 86),
    (5, workgen.OP_PUT, 4096, 1001, 333, 52),
    (7, workgen.OP_PUT, 1 << 20, 3, 3, 40),
    (16, workgen.OP_GET, 4096, 300, 300, 16),
    (1, workgen.OP_PUT, 1 << 16, 300, 300, 256),
    (2, workgen.OP_GET, 4096, 2048, 5, 128),             # exactly one ring's worth of tasks per workgroup
    (8, workgen.OP_PUT, 4096, 4096, 64, 32),             # from here on: enough blocks of four tasks per workgroup
    (8, workgen.OP_GET, 16384, 1024, 1024, 64),          # for the task list to be handed out dynamically
    (4, workgen.OP_PUT, 12288, 2048, 100, 64),           # three tasks per message: blocks straddle messages and slots
    (8, workgen.OP_GET, 1 << 20, 8, 8, 256),
    (2, workgen.OP_PUT, 8192, 4100, 4100, 128),          # 8200 tasks, 128 workgroups per team
    (8, workgen.OP_PUT, 1024, 8192, 500, 32),            # from here on: whole 1 KiB rows that are not whole 4 KiB tasks
    (8, workgen.OP_GET, 3072, 4096, 4096, 64),           # three rows per message: a task straddles messages
    (8, workgen.OP_PUT, 14336, 1024, 300, 256),          # the 14,336-byte token: fourteen rows
    (4, workgen.OP_GET, 5120, 2048, 77, 64),
    (8, workgen.OP_PUT, 2048, 8190, 8190, 32),           # rows not a multiple of sixteen: the last block is short
    (8, workgen.OP_GET, 14336, 301, 301, 64),            # 4214 rows: six rows in the last block; two of the last task's rows are none
    (4, workgen.OP_PUT, 1024, 8195, 1000, 64),           # an odd number of rows
    (8, workgen.OP_PUT, 512, 8192, 1000, 32),            # from here on: several messages to a row
    (8, workgen.OP_GET, 256, 16400, 500, 64),            # 4100 rows: the last block is short
    (4, workgen.OP_PUT, 256, 32776, 4096, 64),
    (4, workgen.OP_PUT, 128, 65544, 4096, 64),           # register path: too short for the streaming kernel to pay
    (8, workgen.OP_GET, 256, 16400, 500, 128),           # the same
    (8, workgen.OP_GET, 512, 8200, 8200, 256),
    (8, workgen.OP_PUT, 256, 16384, 1001, 32),           # the slots are no whole groups: register path
    (8, workgen.OP_PUT, 2048, 1000, 1000, 32),           # too few rows to claim, and no whole 4 KiB tasks: not streamed
    (8, workgen.OP_PUT, 14352, 600, 600, 64),            # the 14,352-byte dispatch message: fourteen rows and 16 bytes
    (8, workgen.OP_GET, 4080, 4100, 999, 32),            # a last row 16 bytes short
    (4, workgen.OP_GET, 1952, 9000, 9000, 64),           # two rows, the second 928 bytes
    (4, workgen.OP_PUT, 1040, 9000, 9000, 64),           # 16 bytes into a second row: too wasteful to stream
    (8, workgen.OP_PUT, 4096, 4099, 4099, 32),           # whole tasks, but not whole blocks of four: claimed as rows
]


def _stream_threads(npes, count, nops, dynamic=True, nslots=None, wgs=0):
    """Workgroup size the library is expected to choose for a streaming cell: 448 (a seventh wave that claims the
    work) either for whole 4 KiB tasks in whole blocks of four, at least eight blocks per workgroup, or for 1 KiB
    rows when the messages fill at least nine tenths of their rows and the PE's rows make at least eight blocks of
    sixteen per workgroup, or for messages of 512 bytes (256 bytes when fewer than 128 workgroups per PE are asked
    for) in whole groups of one row with as many rows;
    else 384 (fixed shares of 4 KiB tasks, at least sixteen per workgroup); 256 for cells that do not stream."""
    if count % 16:
        return 256
    team, rpo, whole, ntasks = 256 // npes, (count + 1023) // 1024, count % 4096 == 0, count // 4096 * nops
    rows = rpo * nops
    claiming = dynamic and team > 1
    if count in (128, 256, 512):
        per_row = 1024 // count
        ok = claiming and (count == 512 or (count == 256 and wgs < 128)) and nops % per_row == 0 and (nslots or nops) % per_row == 0 and nops // per_row // 16 >= 8 * team
        return 448 if ok else 256
    if whole and claiming and ntasks % 4 == 0 and ntasks // 4 >= 8 * team:
        return 448
    if claiming and count * 10 >= rpo * 1024 * 9 and rows // 16 >= 8 * team:
        return 448
    return 384 if whole and ntasks >= 16 * team else 256


@pytest.mark.parametrize("dynamic", [True, False])
@pytest.mark.parametrize("case", STREAM_CASES)
def test_copy_sweep_streaming_cell(case, dynamic, monkeypatch):
    npes, kind, count, nops, nslots, wgs = case
    if not dynamic:
        if _stream_threads(npes, count, nops, True, nslots, wgs) != 448:
            pytest.skip("this cell has a fixed task assignment anyway")
        monkeypatch.setenv("MI_SHMEM_STREAM_DYNAMIC", "0")        # read by shmem_init
    rslot = count + 4096 + 256
    lslot = count + 16
    hb = ((rslot + lslot) * nslots + 8192 + 255) // 256 * 256
    init = seeded_heaps(npes, hb, 1300 + npes + count % 89)
    w = oracle_world(init)
    local_off, remote_off = 16, (lslot * nslots + 16 + 255) // 256 * 256 + 32
    for p in range(npes):
        peer = (p + 1) % npes
        for k in range(nops):
            s = k % nslots
            lo, ro = local_off + s * lslot, remote_off + s * rslot
            rc = w.put(p, ro, lo, count, peer) if kind == workgen.OP_PUT else w.get(p, lo, ro, count, peer)
            assert rc == 0
    w.barrier_all()
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        wgs_launched, threads = sh.copy_sweep_geometry(kind, base + remote_off, base + local_off, count, rslot, lslot, nslots,
                                                       nops, wgs)
        assert threads == _stream_threads(npes, count, nops, dynamic, nslots, wgs)
        assert wgs_launched == (npes * (256 // npes) if threads != 256 else npes * wgs)
        sh.copy_sweep(kind, base + remote_off, base + local_off, count, 1, 1, 1, rslot, lslot, nslots, nops, wgs)
        sh.stream_sync()
        got = heaps_of(heap, npes)
        assert np.array_equal(got, w.heaps())
        assert not np.array_equal(got, init)
        # the claim counters are back at zero: the same cell again, from the same start, gives the same heap
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        sh.copy_sweep(kind, base + remote_off, base + local_off, count, 1, 1, 1, rslot, lslot, nslots, nops, wgs)
        sh.stream_sync()
        assert np.array_equal(heaps_of(heap, npes), w.heaps())


def test_copy_sweep_geometry_keeps_small_cells_on_the_register_path():
    with shmem_world(8, 1 << 22) as (heap, base):
        half = 1 << 21
        assert sh.copy_sweep_geometry(workgen.OP_PUT, base + half, base, 4096, 4096, 4096, 64, 64, 16) == (128, 256)     # under one workgroup per CU
        assert sh.copy_sweep_geometry(workgen.OP_PUT, base + half, base, 4096, 4096, 4096, 64, 64, 32) == (256, 256)     # too few tasks
        assert sh.copy_sweep_geometry(workgen.OP_PUT, base + half, base, 4112, 4352, 4352, 64, 640, 32) == (256, 256)    # not whole tasks
        assert sh.copy_sweep_geometry(workgen.OP_PUT, base + half, base, 4096, 4096, 4096, 64, 640, 32) == (256, 384)     # 20 tasks per workgroup: fixed shares
        assert sh.copy_sweep_geometry(workgen.OP_PUT, base + half, base, 4096, 4096, 4096, 64, 1024, 32) == (256, 448)    # 32 per workgroup: claimed in blocks
        assert sh.copy_sweep_geometry(workgen.OP_IPUT, base + half, base, 4096, 4096 * 8, 4096 * 8, 4, 640, 32) == (256, 256)


@pytest.mark.parametrize("nbytes", [32 << 20, (32 << 20) + 4096 + 48, (40 << 20) + 8])
def test_large_standalone_put_and_get_stream(nbytes):
    """Stand-alone copies of 32 MiB and more: whole 4 KiB tasks through the streaming copy, the rest generic."""
    npes = 2
    hb = ((2 * nbytes + 8192) + 255) // 256 * 256
    init = seeded_heaps(npes, hb, 77 + nbytes % 13)
    w = oracle_world(init)
    src_off, dst_off = 16, (nbytes + 16 + 255) // 256 * 256 + 16
    assert w.put(0, dst_off, src_off, nbytes, 1) == 0
    w.barrier_all()
    assert w.get(1, src_off, dst_off, nbytes, 0) == 0
    w.barrier_all()
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        sh.put(0, base + dst_off, base + src_off, nbytes, 1)
        sh.get(1, base + hb + src_off, base + dst_off, nbytes, 0)
        sh.stream_sync()
        got = heaps_of(heap, npes)
    assert np.array_equal(got, w.heaps())


def test_allocator_matches_oracle_and_host_errors():
    npes, hb = 2, 64 * 256
    w = oracle.World(npes, hb, oracle.EAGER, 0)
    rng = np.random.default_rng(11)
    with shmem_world(npes, hb) as (heap, base):
        assert sh.n_pes() == npes
        live = []
        for step in range(200):
            if live and rng.random() < 0.45:
                off = live.pop(int(rng.integers(0, len(live))))
                assert w.free(off) == 0
                sh.free(base + off)
            else:
                n = int(rng.integers(1, 2000))
                exp = w.malloc(n)
                got = sh.malloc(n)
                assert (got is None) == (exp < 0)
                if got is not None:
                    assert got - base == exp            # same policy, same offsets
                    assert sh.ptr(got, 1) == got + hb
                    live.append(exp)
        assert sh.malloc(0) is None and sh.align(3, 8) is None
        for call, status in [
            (lambda: sh.free(base + 128), sh.ERR_BAD_FREE),
            (lambda: sh.put(0, base, base, 8, 2), sh.ERR_INVALID_PE),
            (lambda: sh.put(-1, base, base, 8, 0), sh.ERR_INVALID_PE),
            (lambda: sh.put(0, base + hb - 4, base, 8, 1), sh.ERR_OUT_OF_RANGE),
            (lambda: sh.get(0, base, base + hb, 1, 1), sh.ERR_OUT_OF_RANGE),
            (lambda: sh.iput(0, base, base, 0, 1, 4, 4, 1), sh.ERR_INVALID_ARG),
            (lambda: sh.iput(0, base + 2, base, 1, 1, 4, 4, 1), sh.ERR_ALIGN),
            (lambda: sh.iput(0, base, base, hb // 4, 1, 2, 4, 1), sh.ERR_OUT_OF_RANGE),
            (lambda: sh.atomic_fetch_add(0, base + 4, 1, 1), sh.ERR_ALIGN),
            (lambda: sh.op_batch(base, 1, 1, 0), sh.ERR_INVALID_ARG),
            (lambda: sh.op_batch(base, 1, 1, 100000), sh.ERR_INVALID_ARG),   # cannot be co-resident
            (lambda: sh.copy_sweep(0, base, base, 64, 1, 1, 1, 256, 256, 1, 1, 1), sh.ERR_INVALID_ARG),
            # a team size whose grid would not fit 32 bits (or any sane launch) is refused, not truncated
            (lambda: sh.copy_sweep(0, base + 4096, base, 64, 1, 1, 1, 256, 256, 1, 1, 2**31 - 1), sh.ERR_INVALID_ARG),
            (lambda: sh.init(2, hb, heap, heap), sh.ERR_ALREADY_INIT),
        ]:
            with pytest.raises(sh.ShmemError) as e:
                call()
            assert e.value.status == status
        assert sh.ptr(base + hb, 0) is None and sh.ptr(base, 2) is None


def test_put_signal_matches_put_then_signal_add():
    # the paper's put with a SignalAdd action as one stream-ordered call: random sizes (zero included: the
    # zero-byte put + signal) and values, several initiators adding to the same signal word
    npes, hb = 4, 1 << 18
    init = seeded_heaps(npes, hb, 4242)
    init[:, hb - 256:] = 0                                   # the signal words start at zero
    w = oracle_world(init)
    sig = hb - 256
    rng = np.random.default_rng(8)
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        for k in range(24):
            me, pe = int(rng.integers(0, npes)), int(rng.integers(0, npes))
            n = int(rng.choice([0, 1, 8, 100, 3000, 4000]))
            lo = k * 8192 + int(rng.integers(0, 64))                       # every op works inside its own 8 KiB stripe
            so = k * 8192 + 4096 + int(rng.integers(0, 64))
            value, word = int(rng.integers(1, 1000)), sig + 8 * int(rng.integers(0, 3))
            assert w.put(me, so, lo, n, pe) == 0
            assert w.signal_add(me, word, value, pe) == 0
            sh.put_signal(me, base + so, sh.ptr(base + lo, me), n, base + word, value, pe)
        sh.barrier_all()
        w.barrier_all()
        assert np.array_equal(heaps_of(heap, npes), w.heaps())
        assert heaps_of(heap, npes)[:, sig:sig + 24].view(np.uint64).sum() > 0
        # host-visible errors enqueue nothing: a bad signal address stops the put as well
        before = heaps_of(heap, npes).copy()
        for call, status in [(lambda: sh.put_signal(0, base, sh.ptr(base + 4096, 0), 64, base + sig + 4, 1, 1), sh.ERR_ALIGN),
                             (lambda: sh.put_signal(0, base, sh.ptr(base + 4096, 0), 64, base + hb, 1, 1), sh.ERR_OUT_OF_RANGE),
                             (lambda: sh.put_signal(0, base + hb - 8, sh.ptr(base, 0), 64, base + sig, 1, 1), sh.ERR_OUT_OF_RANGE),
                             (lambda: sh.put_signal(0, base, sh.ptr(base + 4096, 0), 64, base + sig, 1, npes), sh.ERR_INVALID_PE)]:
            with pytest.raises(sh.ShmemError) as e:
                call()
            assert e.value.status == status
        sh.stream_sync()
        assert np.array_equal(heaps_of(heap, npes), before)

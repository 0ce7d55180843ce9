"""The stream-ordered entry points under HIP graph capture: they only launch kernels on the library's
stream (no allocation, no copy, no synchronisation), so a captured sequence must replay, any number of
times and with eager work between the replays, to the result the same calls give eagerly -- which is the
oracle's.  Serving loops use this to pay one launch for a whole dispatch + combine or a whole table."""
import numpy as np
import pytest
import torch

import oracle
import workgen

pytestmark = pytest.mark.gpu

sh = pytest.importorskip("paper_2511_15076_amd")
import test_gpu_moe as t_moe  # noqa: E402
from gpu_util import heaps_of, shmem_world, to_dev  # noqa: E402
from test_gpu_putget import seeded_heaps  # noqa: E402


def test_table_amo_barrier_sequence_replays_like_eager():
    npes, table_bytes, T, n = 4, 1 << 20, 1024, 50000
    hb = table_bytes + (1 << 16)                           # the table works below 1 MiB, the counters sit above
    ops = workgen.cfg1_op_table()                          # 10,000 puts / gets on 4 PEs, windows of 100
    pe, idx, a = workgen.cfg3_amo_ops(n=n, npes=npes, T=T, dist="zipf", addend="rand16")
    init = seeded_heaps(npes, hb, 1234)
    init[:, table_bytes:] = 0
    w = oracle.World(npes, hb, oracle.SHUFFLED, 9)
    for p in range(npes):
        w.heap(p)[:] = init[p]
    assert w.op_batch(ops, 100) == 0
    w.amo_batch(oracle.AMO_FETCH_ADD, table_bytes, pe, idx, a)
    w.barrier_all()
    want = w.heaps().copy()

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        with shmem_world(npes, hb) as (heap, base):        # the library launches on `stream`
            d_init = torch.from_numpy(init.reshape(-1)).to("cuda:0")
            d_ops, d_pe, d_idx, d_a = to_dev(ops), to_dev(pe), to_dev(idx), to_dev(a)
            d_old = torch.zeros(n, dtype=torch.int64, device="cuda:0")

            def sequence():
                sh.op_batch(d_ops, len(ops), 100, 2)
                sh.amo_batch(sh.AMO_FETCH_ADD, base + table_bytes, T, d_pe, d_idx, d_a, None, d_old, n, 3, 0)
                sh.barrier_all()

            heap.copy_(d_init)
            sequence()                                     # eager
            sh.stream_sync()
            assert np.array_equal(heaps_of(heap, npes), want)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                sequence()
            for replay in range(4):
                heap.copy_(d_init)                         # eager work between the replays
                d_old.zero_()
                sh.put(0, base + table_bytes + 8192, sh.ptr(base, 0), 4096, 1)   # an eager library call, overwritten below
                heap.copy_(d_init)
                graph.replay()
                sh.stream_sync()                           # also reads the device fault word
                assert np.array_equal(heaps_of(heap, npes), want), replay
            del graph


def test_moe_dispatch_combine_replays_like_eager():
    P, E, T, K, Hb, wgs = 4, 16, 16, 4, 272, 3
    topk, ntok = workgen.moe_routing(321, P, E, T, K, ntok=[16, 0, 7, 16], dist="zipf", drop=0.2)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        with shmem_world(P, t_moe.heap_bytes_for(P, E, T, K, Hb)):
            dm = t_moe.DevMoe(P, E, T, K, Hb)
            d_topk, d_ntok = (torch.from_numpy(np.ascontiguousarray(v)).to("cuda:0") for v in (topk, ntok))
            d_x = torch.zeros((P, T, Hb), dtype=torch.uint8, device="cuda:0")
            graph = torch.cuda.CUDAGraph()

            def sequence():                                # identity experts: the received rows go straight back
                sh.moe_dispatch(dm.moe, d_x, d_topk, d_ntok, dm.recv_x, dm.recv_info, dm.recv_range, dm.recv_count, wgs)
                sh.moe_combine(dm.moe, dm.recv_x, dm.recv_info, dm.recv_range, d_topk, d_ntok, dm.combined, wgs)

            sequence()                                     # eager warm-up (epoch 1)
            sh.stream_sync()
            with torch.cuda.graph(graph, stream=stream):
                sequence()
            for replay in range(4):                        # fresh tokens per replay: the graph reads them from d_x
                x = workgen.moe_tokens(700 + replay, P, T, Hb)
                want = t_moe.oracle_run(P, E, T, K, Hb, x, topk, ntok)[0]
                d_x.copy_(torch.from_numpy(x).to("cuda:0"))
                dm.combined.zero_()
                graph.replay()
                sh.stream_sync()
                got = tuple(t.cpu().numpy() for t in (dm.recv_x, dm.recv_info, dm.recv_range, dm.recv_count))
                assert np.array_equal(got[3], want[0][3]) and np.array_equal(got[2], want[0][2])
                for r in range(P):
                    for le in range(E // P):
                        c = want[0][3][r, le]
                        assert np.array_equal(got[0][r, le, :c], want[0][0][r, le, :c])
                        assert np.array_equal(got[1][r, le, :c], want[0][1][r, le, :c])
                assert np.array_equal(dm.combined.cpu().numpy(), want[2]), replay
            del graph
            dm.close()


def test_every_stream_ordered_entry_point_replays_to_its_eager_result():
    # One sequence through the single operations, the sweeps, the hash table, the transpose and the
    # persistent in-kernel exchanges, each in a region of its own.  What the calls give eagerly is held
    # against the oracle by the other test files; here the captured sequence must give the same bytes again.
    npes, hb = 4, 1 << 20
    K = 64 << 10                                           # one 64 KiB region per step
    init = seeded_heaps(npes, hb, 4321)
    n_keys, slots = 600, 256
    keys = workgen.cfg4_keys(n=n_keys)
    queries = workgen.cfg4_queries(keys, n=2 * n_keys)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        with shmem_world(npes, hb) as (heap, base):
            d_init = torch.from_numpy(init.reshape(-1)).to("cuda:0")
            assert sh.malloc(14 * K) == base               # the regions below
            gin = sh.gin_create(2, 1)
            teams = [sh.team_create(0, 2, 2), sh.team_create(1, 2, 2)]          # PEs 0, 2 and PEs 1, 3
            team_words = [sh.team_device_state(t).words_off for t in teams]
            d_keys, d_queries = to_dev(keys), to_dev(queries)
            d_status = torch.zeros(n_keys, dtype=torch.uint8, device="cuda:0")
            d_found = torch.zeros(2 * n_keys, dtype=torch.uint8, device="cuda:0")
            d_old = torch.zeros(4, dtype=torch.int64, device="cuda:0")
            d_err = torch.zeros(1, dtype=torch.int64, device="cuda:0")
            R = [base + i * K for i in range(14)]
            n_t = 64                                       # transpose: 64 x 64 uint32 over 4 PEs = 4 KiB per PE

            def sequence():
                sh.put(0, R[1], sh.ptr(R[0], 0), 5000, 2)
                sh.get(3, sh.ptr(R[1] + 8192, 3), R[0] + 3, 4097, 1)
                sh.fence(0)
                sh.iput(1, R[2], sh.ptr(R[0], 1), 3, 2, 1000, 4, 0)
                sh.iget(2, sh.ptr(R[2] + 32768, 2), R[0], 1, 5, 700, 8, 3)
                sh.quiet()
                sh.atomic_fetch_add(0, R[3], 5, 1, d_old[0:1])
                sh.atomic_compare_swap(1, R[3] + 8, 0, 77, 2, d_old[1:2])
                sh.atomic_fetch_or(2, R[3] + 16, 0xF0, 3, d_old[2:3])
                sh.copy_sweep(sh.OP_PUT, R[5], R[4], 1040, 1, 1, 1, 1280, 1280, 8, 24, 3)
                sh.copy_sweep(sh.OP_IGET, R[7], R[6], 500, 4, 3, 1, 6144, 2304, 4, 9, 2)
                sh.hash_insert(R[8], slots, d_keys, n_keys, d_status, 2)
                sh.hash_lookup(R[8], slots, d_queries, 2 * n_keys, d_found, 2)
                sh.transpose(R[10], R[9], n_t, 4, 2)
                sh.ring_exchange(R[12], R[11], 1000, gin, 1, 0, 3, 2)
                sh.barrier_epochs(R[13], 50, 3, d_err)
                sh.put_signal(1, R[1] + 32768, sh.ptr(R[0], 1), 3000, R[3] + 64, 3, 0)
                sh.team_epochs(teams, [20, 35], R[13] + 1024, 2, d_err)
                sh.team_sync(teams[1], 2)
                sh.barrier_all()

            def start_over():
                heap[:npes * hb].copy_(d_init)
                for p in range(npes):                      # an empty hash table, and what gin_create had cleared
                    heap[p * hb + 8 * K: p * hb + 9 * K].zero_()
                    heap[p * hb + 14 * K: (p + 1) * hb].zero_()
                d_old.zero_(); d_status.fill_(255); d_found.fill_(255)

            def snapshot():
                sh.stream_sync()
                h = heaps_of(heap, npes).copy()
                table = np.sort(h[:, 8 * K: 8 * K + 8 * slots].view(np.uint64), axis=1)   # who won which slot may differ
                h[:, 8 * K: 9 * K] = 0
                for off in team_words:                     # the teams' generation words count barriers: the library's own
                    h[:, off:off + 256] = 0
                return (h, table, d_old.cpu().numpy().copy(), np.sort(d_status.cpu().numpy()), d_found.cpu().numpy().copy(),
                        int(d_err.item()))

            start_over()
            sequence()
            eager = snapshot()
            assert eager[5] == 0 and eager[4].sum() > 0 and not np.array_equal(eager[0], init)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                sequence()
            for replay in range(3):
                start_over()
                graph.replay()
                again = snapshot()
                for k, (x, y) in enumerate(zip(eager, again)):
                    assert np.array_equal(x, y), (replay, k)
            del graph
            for t in teams:
                sh.team_destroy(t)
            sh.gin_destroy(gin)

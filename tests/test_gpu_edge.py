"""Degenerate inputs through the C ABI: every entry point accepts an empty job, enqueues nothing
that touches the heap, and leaves the library usable (OpenSHMEM: a transfer of zero elements is a
no-op, not an error).  Also: set-up with buffers that are too short, and the import order."""
import gc
import os
import subprocess
import sys

import numpy as np
import pytest
import torch

import paper_2511_15076_amd as sh
import workgen
from gpu_util import dev_u8, heaps_of, shmem_world, to_dev

pytestmark = pytest.mark.gpu


def test_empty_jobs_are_no_ops():
    npes, hb = 3, 1 << 16
    init = np.stack([workgen.random_words(900 + p, hb // 8).view(np.uint8) for p in range(npes)])
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        a, b = sh.malloc(4096), sh.malloc(4096)
        # single operations of zero elements (a null local pointer is fine when nothing is moved)
        sh.put(0, a, sh.ptr(b, 0), 0, 1)
        sh.put(0, a, None, 0, 1)
        sh.get(2, sh.ptr(b, 2), a, 0, 0)
        sh.get(2, sh.ptr(b, 2), a + 4096, 0, 0)          # one past the end of an object, zero bytes: in range
        sh.iput(0, a, sh.ptr(b, 0), 1, 1, 0, 4, 1)
        sh.iget(1, sh.ptr(b, 1), a, 3, 2, 0, 8, 2)
        # tables, sweeps and batches with nothing in them
        sh.op_batch(None, 0, 0, 1)
        sh.op_batch(None, 0, 7, 4)
        sh.copy_sweep(sh.OP_PUT, a, b, 0, 1, 1, 1, 0, 0, 1, 5, 2)        # zero-byte messages
        sh.copy_sweep(sh.OP_IGET, a, b, 16, 4, 2, 2, 0, 0, 1, 0, 2)      # zero ops per PE
        sh.amo_batch(sh.AMO_FETCH_ADD, a, 16, None, None, None, None, None, 0, 2)
        sh.amo_batch(sh.AMO_COMPARE_SWAP, a, 16, None, None, None, None, None, 0, 2, 1)
        sh.hash_insert(a, 16, None, 0, None, 2)
        sh.hash_lookup(a, 16, None, 0, None, 2)
        sh.transpose(a, b, 0, 4, 2)
        sh.fence(0)
        sh.quiet()
        sh.barrier_all()
        sh.stream_sync()
        assert np.array_equal(heaps_of(heap, npes), init)

        # objects: zero rounds, zero iterations, zero descriptors
        gin = sh.gin_create(2, 1)
        sh.ring_exchange(a, b, 256, gin, 0, 0, 0, 2)
        sh.ring_exchange(a, b, 0, gin, 0, 0, 3, 2)                       # three rounds of empty slots
        sh.pingpong(a, 0, gin, 1, 0)
        sh.pingpong(a, 0, gin, 1, 4)                                     # signals only
        sh.barrier_epochs(a, 0, 2)
        proxy = sh.proxy_create(8)
        sh.proxy_submit(proxy, None, 0, 2)
        sh.proxy_quiet(proxy)
        assert sh.proxy_stats(proxy) == {"submitted": 0, "executed": 0, "rejected": 0}
        sh.proxy_destroy(proxy)
        sh.stream_sync()
        got = heaps_of(heap, npes)
        lo = a - base
        assert np.array_equal(got[:, lo:lo + 8192], init[:, lo:lo + 8192])   # both objects untouched on every PE
        sh.gin_destroy(gin)

        # and the library still works
        sh.put(0, a, sh.ptr(b, 0), 4096, 1)
        sh.stream_sync()
        assert np.array_equal(heaps_of(heap, npes)[1, lo:lo + 4096], init[0, lo + 4096:lo + 8192])


def test_bfs_on_graphs_without_edges():
    # a single vertex, and several isolated vertices: one level, the root alone, nothing traversed
    for nverts, npes, root in [(1, 1, 0), (5, 2, 3), (130, 3, 129)]:
        with shmem_world(npes, 1 << 20):
            row_off = to_dev(np.zeros(nverts + 1, dtype=np.uint64))
            nbr = dev_u8(16)
            for mode in (sh.BFS_TOP_DOWN, sh.BFS_DIRECTION_OPTIMIZING, sh.BFS_BOTTOM_UP | sh.BFS_CANONICAL_PARENTS):
                g = sh.bfs_create(nverts, row_off, nbr, 2)
                sh.bfs_configure(g, mode)
                level = torch.zeros(nverts, dtype=torch.int32, device="cuda:0")
                parent = torch.zeros(nverts, dtype=torch.int32, device="cuda:0")
                st = sh.bfs(g, root, level, parent)
                sh.stream_sync()
                want_level = np.full(nverts, -1, dtype=np.int32)
                want_level[root] = 0
                want_parent = np.full(nverts, sh.BFS_NONE, dtype=np.uint32)
                want_parent[root] = root
                assert np.array_equal(level.cpu().numpy(), want_level)
                assert np.array_equal(parent.cpu().numpy().view(np.uint32), want_parent)
                assert (st["nlevels"], st["reached"], st["edges_traversed"], st["frontier_size"]) == (1, 1, 0, [1])
                sh.bfs_destroy(g)


def test_bfs_create_refuses_a_broken_graph():
    # a neighbour that is no vertex, and row offsets that decrease: refused when the graph is created (the library
    # rewrites the adjacency in its own numbering then, so it sees every entry), nothing left allocated
    with shmem_world(2, 1 << 20) as (heap, base):
        row = np.array([0, 2, 3, 4, 4], dtype=np.uint64)
        for nbr, r in ((np.array([1, 2, 0, 9], dtype=np.uint32), row),              # 9 is no vertex of a graph of 4
                       (np.array([1, 2, 0, 0], dtype=np.uint32), np.array([0, 2, 1, 4, 4], dtype=np.uint64))):
            with pytest.raises(sh.ShmemError) as ei:
                sh.bfs_create(4, to_dev(r), to_dev(nbr), 1)
            assert ei.value.status == sh.ERR_INVALID_ARG
        assert sh.malloc(1 << 20) == base                  # the per-PE state went back to the heap
        sh.free(base)
        g = sh.bfs_create(4, to_dev(row), to_dev(np.array([1, 2, 0, 0], dtype=np.uint32)), 1)   # the library still works
        assert sh.bfs(g, 0)["reached"] == 3
        sh.bfs_destroy(g)


def test_init_rejects_buffers_shorter_than_stated():
    # with torch's cache emptied, an allocation of 16 MiB is a block of its own and the runtime knows where it ends
    def status_of(*args):
        try:
            sh.init(*args)
        except sh.ShmemError as e:
            return e.status
        sh.finalize()
        return sh.OK

    dev = torch.device("cuda:0")
    gc.collect()                                                 # no stale tensor keeps a cached segment alive
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    heap = torch.zeros(16 << 20, dtype=torch.uint8, device=dev)
    big = torch.zeros(16 << 20, dtype=torch.uint8, device=dev)
    scratch = torch.zeros(sh.scratch_bytes(4), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    assert status_of(4, 16 << 20, heap, scratch, stream) == sh.ERR_OUT_OF_RANGE             # four segments claimed, one provided
    assert status_of(4, 4 << 20, heap.data_ptr() + 256, scratch, stream) == sh.ERR_OUT_OF_RANGE   # the last segment ends 256 bytes late
    assert status_of(4, 4 << 20, heap, big.data_ptr() + (16 << 20) - 256, stream) == sh.ERR_OUT_OF_RANGE   # scratch words: 256 bytes left
    assert status_of(4, 4 << 20, heap, scratch, stream) == sh.OK                             # the exact size is fine


def test_package_imported_before_torch_shares_its_runtime():
    # whichever is imported first, the library and torch must end up on one HIP runtime
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = (
        "import sys; sys.path.insert(0, %r)\n"
        "import paper_2511_15076_amd as sh\n"
        "import torch\n"
        "heap = torch.zeros(2 << 16, dtype=torch.uint8, device='cuda:0')\n"
        "heap[:4096] = 7\n"
        "scratch = torch.zeros(sh.scratch_bytes(2), dtype=torch.uint8, device='cuda:0')\n"
        "sh.init(2, 1 << 16, heap, scratch, torch.cuda.current_stream().cuda_stream)\n"
        "a = sh.malloc(8192)\n"
        "sh.put(0, a + 4096, sh.ptr(a, 0), 4096, 1)\n"
        "sh.stream_sync()\n"
        "assert int(heap[(1 << 16) + 4096:(1 << 16) + 8192].sum()) == 7 * 4096\n"
        "sh.finalize()\n"
        "print('ok')\n") % (root,)
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0 and out.stdout.strip().endswith("ok"), out.stderr[-2000:]

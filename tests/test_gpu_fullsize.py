"""GPU parity at the full sizes of the five configurations, in the launch
configurations that bench.py times.  Where the oracle can afford the whole
workload it is compared bit-exact; otherwise sampled outputs are computed by
the oracle one by one and properties that hold at any size cover the rest."""
import numpy as np
import pytest
import torch

import oracle
import workgen

pytestmark = pytest.mark.gpu

sh = pytest.importorskip("paper_2511_15076_amd")
from gpu_util import as_np, shmem_world, to_dev  # noqa: E402

_cache = {}


@pytest.mark.parametrize("nbytes", [1 << 20, 1 << 26])
def test_config2_bench_cells(nbytes):
    # the cells bench.py times: 8 PEs x 1 GiB, 256 workgroups per PE, 256 MiB of payload per PE
    npes, seg, wgs = 8, 1 << 30, 256
    ops = (1 << 28) // nbytes
    rng = np.random.default_rng(nbytes % 1000)
    with shmem_world(npes, seg) as (heap, base):
        heap.view(torch.int64).random_()
        h = heap.view(npes, seg)
        local, remote = 0, seg // 2
        for kind in (sh.OP_PUT, sh.OP_GET):
            h[:, seg - 4096:].fill_(0x5A)                        # sentinel beyond both windows
            before = h[:, remote - 4096:remote].clone()
            sh.copy_sweep(kind, base + remote, base + local, nbytes, 1, 1, 1, nbytes, nbytes, ops, ops, wgs)
            sh.stream_sync()
            for p in range(npes):
                peer = (p + 1) % npes
                # invariant at any size: after put + quiet the target bytes equal the source
                assert torch.equal(h[peer, remote:remote + (1 << 28)], h[p, local:local + (1 << 28)])
            assert bool((h[:, seg - 4096:] == 0x5A).all())
            if kind == sh.OP_PUT:
                assert torch.equal(h[:, remote - 4096:remote], before)   # bytes below the window untouched
            # sampled windows, each computed by the oracle
            for _ in range(6):
                p = int(rng.integers(0, npes)); peer = (p + 1) % npes
                k = int(rng.integers(0, ops)); ln = int(rng.choice([8, 4096, 65536]))
                a = int(rng.integers(0, (nbytes - ln) // 8 + 1)) * 8
                w = oracle.World(2, 1 << 17, oracle.SHUFFLED, 1)
                src_pe, src_off = (p, local) if kind == sh.OP_PUT else (peer, remote)
                dst_pe, dst_off = (peer, remote) if kind == sh.OP_PUT else (p, local)
                src = h[src_pe, src_off + k * nbytes + a: src_off + k * nbytes + a + ln].cpu().numpy()
                w.heap(0)[:ln] = src
                if kind == sh.OP_PUT:
                    w.put(0, 0, 0, ln, 1); w.quiet(0)
                    exp = w.heap(1)[:ln]
                else:
                    w.heap(1)[:ln] = src
                    w.get(0, 65536, 0, ln, 1)
                    exp = w.heap(0)[65536:65536 + ln]
                got = h[dst_pe, dst_off + k * nbytes + a: dst_off + k * nbytes + a + ln].cpu().numpy()
                assert np.array_equal(got, exp)
            heap.view(torch.int64).random_()                     # fresh payload for the next kind


@pytest.mark.parametrize("nbytes,wgs", [(256, 64), (512, 32), (512, 256), (1024, 64), (14336, 256), (14352, 32)])
def test_config2_sweep_cells_below_1mib(nbytes, wgs):
    # cells of the full sweep that the streaming copy takes in other shapes than whole 4 KiB tasks (several messages
    # to a 1 KiB row; rows with a short last one), at the sweep's own sizes: 65,536 messages per PE (or 256 MiB), every
    # message in its own slot of the next multiple of 256 bytes
    npes, seg = 8, 1 << 30
    slot = (nbytes + 255) // 256 * 256
    ops = min((1 << 28) // nbytes, 1 << 16)
    nslots = max(1, min((seg // 2) // slot, (1 << 28) // slot))
    rng = np.random.default_rng(nbytes)
    with shmem_world(npes, seg) as (heap, base):
        heap.view(torch.int64).random_()
        h = heap.view(npes, seg)
        touched = min(ops, nslots)                              # (the sweep's 14,352-byte cell goes round its slots once)
        local, remote, span = 0, seg // 2, touched * slot
        for kind in (sh.OP_PUT, sh.OP_GET):
            src_off, dst_off = (local, remote) if kind == sh.OP_PUT else (remote, local)
            before = h[:, dst_off:dst_off + span + 4096].clone()
            threads = sh.copy_sweep_geometry(kind, base + remote, base + local, nbytes, slot, slot, nslots, ops, wgs)[1]
            assert threads == 448                                  # the streaming copy with claimed work
            sh.copy_sweep(kind, base + remote, base + local, nbytes, 1, 1, 1, slot, slot, nslots, ops, wgs)
            sh.stream_sync()
            for p in range(npes):
                peer = (p + 1) % npes
                src_pe, dst_pe = (p, peer) if kind == sh.OP_PUT else (peer, p)
                got = h[dst_pe, dst_off:dst_off + span].view(touched, slot)
                assert torch.equal(got[:, :nbytes], h[src_pe, src_off:src_off + span].view(touched, slot)[:, :nbytes])
                if slot > nbytes:                                  # the bytes between the messages are as they were
                    assert torch.equal(got[:, nbytes:], before[dst_pe, :span].view(touched, slot)[:, nbytes:])
                assert torch.equal(h[dst_pe, dst_off + span:dst_off + span + 4096], before[dst_pe, span:])
            for _ in range(6):                                     # sampled messages, each computed by the oracle
                p = int(rng.integers(0, npes)); peer = (p + 1) % npes
                k = int(rng.integers(0, touched))
                src_pe, dst_pe = (p, peer) if kind == sh.OP_PUT else (peer, p)
                w = oracle.World(2, 1 << 16, oracle.SHUFFLED, 1)
                w.heap(0)[:] = 0; w.heap(1)[:] = 0
                w.heap(0 if kind == sh.OP_PUT else 1)[:nbytes] = h[src_pe, src_off + k * slot:src_off + k * slot + nbytes].cpu().numpy()
                if kind == sh.OP_PUT:
                    w.put(0, 32768, 0, nbytes, 1); w.quiet(0)
                    exp = w.heap(1)[32768:32768 + nbytes]
                else:
                    w.get(0, 32768, 0, nbytes, 1)
                    exp = w.heap(0)[32768:32768 + nbytes]
                assert np.array_equal(h[dst_pe, dst_off + k * slot:dst_off + k * slot + nbytes].cpu().numpy(), exp)
            heap.view(torch.int64).random_()


# The strided cells bench.py times: uint32, 4 MiB of payload per op (2^20 elements), 256 workgroups per PE, 8 PEs;
# gather (the read side strided), scatter (the written side strided) and both, at strides 2, 16 and 64.  The heap is
# random, so every byte between the elements of a strided destination is a sentinel that must survive.
@pytest.mark.parametrize("kind,ls,rs", [(sh.OP_IPUT, 2, 1), (sh.OP_IPUT, 1, 2), (sh.OP_IPUT, 2, 2),
                                        (sh.OP_IPUT, 16, 1), (sh.OP_IPUT, 1, 16), (sh.OP_IPUT, 16, 16),
                                        (sh.OP_IPUT, 64, 1), (sh.OP_IPUT, 1, 64), (sh.OP_IPUT, 64, 64),
                                        (sh.OP_IGET, 1, 2), (sh.OP_IGET, 16, 1), (sh.OP_IGET, 64, 64)])
def test_config2_strided_bench_cells(kind, ls, rs):
    npes, wgs, nelems, ops = 8, 256, (4 << 20) // 4, 2
    lspan, rspan = ((nelems - 1) * ls + 1) * 4, ((nelems - 1) * rs + 1) * 4
    lslot, rslot = (lspan + 255) // 256 * 256, (rspan + 255) // 256 * 256
    nslots = 2 if max(ls, rs) <= 16 else 1                    # the second op of a stride-64 cell works on the same slot again
    local, remote = 256, 256 + nslots * lslot + 4096
    seg = (remote + nslots * rslot + 4096 + 255) // 256 * 256
    init = np.stack([workgen.random_words(4000 + 16 * ls + rs + p, seg // 8).view(np.uint8) for p in range(npes)])
    w = oracle.World(npes, seg, oracle.SHUFFLED, 3)
    for p in range(npes):
        w.heap(p)[:] = init[p]
    for p in range(npes):
        peer = (p + 1) % npes
        for k in range(ops):
            lo, ro = local + (k % nslots) * lslot, remote + (k % nslots) * rslot
            rc = w.iput(p, ro, lo, rs, ls, nelems, 4, peer) if kind == sh.OP_IPUT else w.iget(p, lo, ro, ls, rs, nelems, 4, peer)
            assert rc == 0
    w.barrier_all()
    with shmem_world(npes, seg) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        sh.copy_sweep(kind, base + remote, base + local, nelems, 4, rs, ls, rslot, lslot, nslots, ops, wgs)
        sh.stream_sync()
        got = heap.cpu().numpy().reshape(npes, seg)
    assert np.array_equal(got, w.heaps())
    assert not np.array_equal(got, init)
    w.close()


@pytest.mark.parametrize("dist,T,agg", [("uniform", 1, 1), ("zipf", 1024, 0), ("uniform", 1 << 20, 0),
                                        ("zipf", 1 << 20, 1)])
def test_config3_full(dist, T, agg):
    npes, n, seg, wgs = 64, 1 << 24, 8 << 20, 32
    pe, idx, a = workgen.cfg3_amo_ops(n=n, npes=npes, T=T, dist=dist, addend="rand16")
    tag = np.arange(1, n + 1, dtype=np.uint64)
    w = oracle.World(npes, seg, oracle.AT_QUIET, 0)
    off = w.malloc(T * 8)
    w.amo_batch(oracle.AMO_FETCH_ADD, off, pe, idx, a)
    exp_add = np.stack([w.heap(p)[off:off + 8 * T].view(np.uint64).copy() for p in range(npes)])
    for p in range(npes):
        w.heap(p)[off:off + 8 * T] = 0
    w.amo_batch(oracle.AMO_COMPARE_SWAP, off, pe, idx, np.zeros(n, np.uint64), tag)
    exp_claimed = np.stack([w.heap(p)[off:off + 8 * T].view(np.uint64) != 0 for p in range(npes)])
    for p in range(npes):
        w.heap(p)[off:off + 8 * T] = 0
    w.amo_batch(oracle.AMO_MIN_CAS_LOOP, off, pe, idx, tag)
    exp_min = np.stack([w.heap(p)[off:off + 8 * T].view(np.uint64).copy() for p in range(npes)])
    w.close()
    with shmem_world(npes, seg) as (heap, base):
        ctr = sh.malloc(T * 8)
        assert ctr - base == off
        view = heap.view(npes, seg)[:, off:off + 8 * T]
        d_pe, d_idx, d_a, d_tag = to_dev(pe), to_dev(idx), to_dev(a), to_dev(tag)
        d_zero = torch.zeros(n, dtype=torch.int64, device="cuda:0")
        d_old = torch.empty(n, dtype=torch.int64, device="cuda:0")
        sh.amo_batch(sh.AMO_FETCH_ADD, ctr, T, d_pe, d_idx, d_a, None, d_old, n, wgs, agg)
        sh.stream_sync()
        got = view.cpu().numpy().view(np.uint64).reshape(npes, T)
        assert np.array_equal(got, exp_add)
        old = as_np(d_old, np.uint64)
        key = pe.astype(np.int64) * T + idx                      # permutation of prefix sums, every counter
        order = np.lexsort((old, key))
        k, f, aa = key[order], old[order], a[order]
        first = np.r_[True, k[1:] != k[:-1]]
        assert (f[first] == 0).all()
        assert np.array_equal(f[1:][~first[1:]], (f[:-1] + aa[:-1])[~first[1:]])
        view.zero_()
        sh.amo_batch(sh.AMO_COMPARE_SWAP, ctr, T, d_pe, d_idx, d_zero, d_tag, d_old, n, wgs, 0)
        sh.stream_sync()
        got = view.cpu().numpy().view(np.uint64).reshape(npes, T)
        assert np.array_equal(got != 0, exp_claimed)
        old = as_np(d_old, np.uint64)
        win = old == 0
        assert int(win.sum()) == int(exp_claimed.sum())
        flat = got.reshape(-1)
        assert np.array_equal(flat[key[win]], tag[win]) and np.array_equal(old[~win], flat[key[~win]])
        view.zero_()
        sh.amo_batch(sh.AMO_MIN_CAS_LOOP, ctr, T, d_pe, d_idx, d_tag, None, None, n, wgs, agg)
        sh.stream_sync()
        assert np.array_equal(view.cpu().numpy().view(np.uint64).reshape(npes, T), exp_min)


def _cfg4():
    if "cfg4" not in _cache:
        n, npes = 1 << 26, 16
        keys = workgen.cfg4_keys(n=n)
        queries = workgen.cfg4_queries(keys, n=n)
        _cache["cfg4"] = (n, npes, 2 * n // npes, keys, queries)
    return _cache["cfg4"]


def test_config4_full_insert_and_lookup():
    n, npes, slots, keys, queries = _cfg4()
    seg = slots * 8 + (1 << 20)
    w = oracle.World(npes, seg, oracle.AT_QUIET, 0)
    tab = w.malloc(slots * 8)
    ost = w.hash_insert(tab, slots, keys)
    print("oracle insert done", flush=True)
    nq = 1 << 23                                                  # sampled lookups, one by one in the oracle
    ofound = w.hash_lookup(tab, slots, queries[:nq])
    with shmem_world(npes, seg) as (heap, base):
        t = sh.malloc(slots * 8)
        assert t - base == tab
        dk, dq = to_dev(keys), to_dev(queries)
        dst = torch.full((n,), 255, dtype=torch.uint8, device="cuda:0")
        dfo = torch.full((n,), 255, dtype=torch.uint8, device="cuda:0")
        sh.hash_insert(t, slots, dk, n, dst, 128)
        sh.hash_lookup(t, slots, dq, n, dfo, 128)
        sh.stream_sync()
        st, found = as_np(dst, np.uint8), as_np(dfo, np.uint8)
        assert np.array_equal(st, ost)                            # no duplicates here: every status unique
        assert np.array_equal(found[:nq], ofound)
        assert abs(float(found.mean()) - 0.5) < 1e-3 and set(np.unique(found)) <= {0, 1}
        view = heap.view(npes, seg)[:, tab:tab + 8 * slots]
        for p in range(npes):
            g = view[p].cpu().numpy().view(np.uint64)
            o = w.heap(p)[tab:tab + 8 * slots].view(np.uint64)
            assert np.array_equal(g != 0, o != 0)                 # occupancy is order-independent
            if p in (0, 7):
                assert np.array_equal(np.sort(g), np.sort(o))     # same keys stored on this PE


def test_config5_full_eight_roots():
    scale, npes, wgs = 24, 16, 64
    n = 1 << scale
    row, nbr = workgen.rmat_csr(scale)
    print("graph built", flush=True)
    roots = workgen.bfs_roots(row, 64)[[0, 5, 13, 22, 37, 41, 56, 63]]          # 8 of the 64 roots bench.py times
    vpp = n // npes
    seg = ((vpp * 28 + vpp // 8 + (1 << 16)) + 255) // 256 * 256
    w = oracle.World(npes, seg, oracle.AT_QUIET, 0)
    deg = np.diff(row).astype(np.int64)
    with shmem_world(npes, seg) as (heap, base):
        drow, dnbr = to_dev(row), to_dev(nbr)
        g = sh.bfs_create(n, drow, dnbr, wgs)
        dl = torch.empty(n, dtype=torch.int32, device="cuda:0")
        dp = torch.empty(n, dtype=torch.int32, device="cuda:0")
        for root in roots:
            olevel, oparent, ostats = w.bfs(row, nbr, int(root))
            print("oracle search done", flush=True)
            for mode in (sh.BFS_TOP_DOWN, sh.BFS_DIRECTION_OPTIMIZING):
                sh.bfs_configure(g, mode)
                stats = sh.bfs(g, int(root), dl, dp)
                level, parent = as_np(dl, np.int32).copy(), as_np(dp, np.uint32).copy()
                assert np.array_equal(level, olevel)
                assert stats == ostats
                reached = level >= 0
                assert parent[root] == root and ((parent == sh.BFS_NONE) == ~reached).all()
                vs = np.flatnonzero(reached)
                vs = vs[vs != root]
                us = parent[vs].astype(np.int64)
                assert (level[us] == level[vs] - 1).all()             # every tree edge spans one level
                assert stats["edges_traversed"] == int(deg[reached].sum()) // 2
                for v in vs[:: max(1, len(vs) // 2000)]:              # sampled: the tree edge exists
                    u = int(parent[v])
                    assert v in nbr[row[u]:row[u + 1]]
            if root not in (roots[0], roots[4]):
                continue
            # canonical parents at full size: sampled vertices, each computed from the oracle's levels
            sh.bfs_configure(g, sh.BFS_DIRECTION_OPTIMIZING | sh.BFS_CANONICAL_PARENTS)
            sh.bfs(g, int(root), dl, dp)
            parent = as_np(dp, np.uint32).copy()
            reached = olevel >= 0
            assert parent[root] == root and ((parent == sh.BFS_NONE) == ~reached).all()
            vs = np.flatnonzero(reached)
            hubs = np.argsort(deg)[-3:]                               # the longest rows go through the wave-wide scan
            for v in list(vs[:: max(1, len(vs) // 3000)]) + [int(h) for h in hubs if reached[h]]:
                if v == root:
                    continue
                adj = nbr[row[v]:row[v + 1]]
                assert parent[v] == adj[olevel[adj] == olevel[v] - 1].min(), v
        sh.bfs_destroy(g)

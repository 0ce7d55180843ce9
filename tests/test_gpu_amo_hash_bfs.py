"""GPU parity for the atomic path, the hash table and BFS.

Where several results are correct (fetched values, compare-swap winners, slot
placement, BFS parents) the unique part is compared bit-exact with the oracle
and the rest is checked for validity."""
import itertools

import numpy as np
import pytest
import torch

import oracle
import workgen

pytestmark = pytest.mark.gpu

sh = pytest.importorskip("paper_2511_15076_amd")
from gpu_util import as_np, heaps_of, shmem_world, to_dev  # noqa: E402


def counters_of(heap, npes, off, T):
    h = heaps_of(heap, npes)
    return np.stack([h[p][off:off + 8 * T].view(np.uint64) for p in range(npes)])


def run_amo(kind, npes, T, pe, idx, a, b, wgs, agg, hb):
    n = len(pe)
    with shmem_world(npes, hb) as (heap, base):
        ctr = sh.malloc(T * 8)
        d_pe, d_idx, d_a = to_dev(pe), to_dev(idx), to_dev(a)
        d_b = to_dev(b) if b is not None else None
        d_old = torch.zeros(n, dtype=torch.int64, device="cuda:0")
        sh.amo_batch(kind, ctr, T, d_pe, d_idx, d_a, d_b, d_old, n, wgs, agg)
        sh.stream_sync()
        return counters_of(heap, npes, ctr - base, T), as_np(d_old, np.uint64).copy(), ctr - base


def check_prefix_sums(pe, idx, a, old, T):
    key = pe.astype(np.int64) * T + idx
    order = np.lexsort((old, key))
    k, f, aa = key[order], old[order], a[order]
    first = np.r_[True, k[1:] != k[:-1]]
    assert (f[first] == 0).all()
    same = ~first[1:]
    assert np.array_equal(f[1:][same], (f[:-1] + aa[:-1])[same])


@pytest.mark.parametrize("agg", [0, 1])
@pytest.mark.parametrize("dist,T,npes", [("uniform", 1, 64), ("zipf", 1024, 64), ("uniform", 4096, 16),
                                         ("zipf", 37, 5)])
def test_fetch_add_batch(agg, dist, T, npes):
    n = 200000 + 77                                      # several passes and a ragged tail
    hb = max(1 << 16, ((T * 8 + 255) // 256 + 1) * 256)
    for addend in ("one", "rand16"):
        pe, idx, a = workgen.cfg3_amo_ops(n=n, npes=npes, T=T, dist=dist, addend=addend)
        final, old, off = run_amo(sh.AMO_FETCH_ADD, npes, T, pe, idx, a, None, 3, agg, hb)
        w = oracle.World(npes, hb, oracle.SHUFFLED, 0)
        assert w.malloc(T * 8) == off
        oold = w.amo_batch(oracle.AMO_FETCH_ADD, off, pe, idx, a)
        ofinal = np.stack([w.heap(p)[off:off + 8 * T].view(np.uint64) for p in range(npes)])
        assert np.array_equal(final, ofinal)
        check_prefix_sums(pe, idx, a, old, T)            # a permutation of prefix sums
        if addend == "one":                              # per counter the same multiset as the oracle
            key = pe.astype(np.int64) * T + idx
            assert np.array_equal(old[np.lexsort((old, key))], oold[np.lexsort((oold, key))])


@pytest.mark.parametrize("agg", [0, 1])
def test_fetch_or_and_min_loop_batch(agg):
    npes, T, n = 16, 64, 150001
    hb = 1 << 16
    pe, idx, tag = workgen.cfg3_amo_ops(n=n, npes=npes, T=T, dist="zipf", addend="tag")
    bits = (np.uint64(1) << (tag % np.uint64(64))).astype(np.uint64)
    final, old, off = run_amo(sh.AMO_FETCH_OR, npes, T, pe, idx, bits, None, 2, agg, hb)
    w = oracle.World(npes, hb, oracle.SHUFFLED, 0)
    assert w.malloc(T * 8) == off
    w.amo_batch(oracle.AMO_FETCH_OR, off, pe, idx, bits)
    assert np.array_equal(final, np.stack([w.heap(p)[off:off + 8 * T].view(np.uint64) for p in range(npes)]))
    # exactly one op per (word, bit) saw the bit clear
    clear = (old & bits) == 0
    key = (pe.astype(np.int64) * T + idx) * 64 + (tag % np.uint64(64)).astype(np.int64)
    assert len(np.unique(key[clear])) == int(clear.sum()) == len(np.unique(key))
    # min through a compare-swap loop: closed form min per word
    tag = np.random.default_rng(2).permutation(tag)
    final, _, off = run_amo(sh.AMO_MIN_CAS_LOOP, npes, T, pe, idx, tag, None, 2, agg, hb)
    w2 = oracle.World(npes, hb, oracle.SHUFFLED, 0)
    assert w2.malloc(T * 8) == off
    w2.amo_batch(oracle.AMO_MIN_CAS_LOOP, off, pe, idx, tag)
    assert np.array_equal(final, np.stack([w2.heap(p)[off:off + 8 * T].view(np.uint64) for p in range(npes)]))


def _min_loop_values_fit_a_serial_order(a, old):
    """The ops on ONE word (operands a, fetched values old, word initially 0): is there an order in which every
    op fetched what the word held just before it?  The word only changes when an op lowers it (or fills it while
    it is 0), so the order is forced: at value v, first every op that fetched v and leaves it alone, then the one
    op that fetched v and changes it."""
    left = list(zip(a.tolist(), old.tolist()))
    v = 0
    while left:
        here = [(x, o) for x, o in left if o == v]
        if not here:
            return False
        movers = [x for x, o in here if v == 0 or x < v]
        if len(movers) > 1:
            return False
        left = [(x, o) for x, o in left if o != v]
        if movers:
            v = movers[0]
        elif left:
            return False           # nobody moves the word on, yet ops remain that fetched something else
    return True


@pytest.mark.parametrize("agg", [0, 1])
def test_min_loop_fetched_values_fit_a_serial_order(agg):
    # few words, many ops per word, operands with repeats: the combining kernel merges dozens of ops per word
    npes, T, n, hb = 4, 3, 6000, 1 << 12
    rng = np.random.default_rng(17)
    pe = rng.integers(0, npes, n).astype(np.int32)
    idx = rng.integers(0, T, n).astype(np.uint32)
    a = rng.integers(1, 400, n).astype(np.uint64)
    final, old, _ = run_amo(sh.AMO_MIN_CAS_LOOP, npes, T, pe, idx, a, None, 2, agg, hb)
    for p in range(npes):
        for t in range(T):
            m = (pe == p) & (idx == t)
            assert final[p, t] == a[m].min()
            assert _min_loop_values_fit_a_serial_order(a[m], old[m]), (p, t)
    # the checker itself: a dropped dependency must not pass
    assert _min_loop_values_fit_a_serial_order(np.array([5, 3, 7]), np.array([0, 5, 3]))
    assert not _min_loop_values_fit_a_serial_order(np.array([5, 3]), np.array([0, 0]))
    assert not _min_loop_values_fit_a_serial_order(np.array([5, 3, 7]), np.array([0, 5, 7]))
    assert not _min_loop_values_fit_a_serial_order(np.array([5, 3, 2]), np.array([0, 5, 5]))


@pytest.mark.parametrize("dist,T", [("uniform", 1), ("zipf", 1024)])
def test_compare_swap_claim_batch(dist, T):
    npes, n, hb = 64, 120000, 1 << 16
    pe, idx, tag = workgen.cfg3_amo_ops(n=n, npes=npes, T=T, dist=dist, addend="tag")
    zeros = np.zeros(n, dtype=np.uint64)
    final, old, off = run_amo(sh.AMO_COMPARE_SWAP, npes, T, pe, idx, zeros, tag, 2, 0, hb)
    w = oracle.World(npes, hb, oracle.SHUFFLED, 0)
    assert w.malloc(T * 8) == off
    w.amo_batch(oracle.AMO_COMPARE_SWAP, off, pe, idx, zeros, tag)
    ofinal = np.stack([w.heap(p)[off:off + 8 * T].view(np.uint64) for p in range(npes)])
    assert np.array_equal(final != 0, ofinal != 0)       # the set of claimed slots is unique
    key = pe.astype(np.int64) * T + idx
    winners = old == 0
    assert int(winners.sum()) == len(np.unique(key)) == int((final != 0).sum())
    assert len(np.unique(key[winners])) == int(winners.sum())   # one winner per slot
    flat = final.reshape(-1)
    assert np.array_equal(flat[key[winners]], tag[winners])     # the slot holds its winner's tag
    assert np.array_equal(old[~winners], flat[key[~winners]])   # losers saw the final value


def test_compare_swap_outcomes_are_linearisable():
    # tiny programs: every outcome the GPU produces must be reachable by some
    # serial order of the same ops (brute force over all orders)
    rng = np.random.default_rng(8)
    npes, hb = 3, 4096
    for trial in range(12):
        n = int(rng.integers(2, 7))
        slot = rng.integers(0, 2, n)
        cond = rng.integers(0, 3, n).astype(np.uint64)
        val = rng.integers(1, 4, n).astype(np.uint64)
        allowed = set()
        for order in itertools.permutations(range(n)):
            mem, seen = [0, 0], [0] * n
            for i in order:
                seen[i] = mem[slot[i]]
                if mem[slot[i]] == cond[i]:
                    mem[slot[i]] = int(val[i])
            allowed.add((tuple(mem), tuple(seen)))
        pe = np.full(n, 2, dtype=np.int32)               # all target PE 2; issuers spread over the PEs
        for rep in range(4):
            final, old, off = run_amo(sh.AMO_COMPARE_SWAP, npes, 2, pe, slot.astype(np.uint32), cond, val,
                                      1, 0, hb)
            got = (tuple(int(x) for x in final[2]), tuple(int(x) for x in old))
            assert got in allowed, (trial, got)


def test_single_amos():
    npes, hb = 4, 4096
    w = oracle.World(npes, hb, oracle.SHUFFLED, 0)
    with shmem_world(npes, hb) as (heap, base):
        res = torch.zeros(8, dtype=torch.int64, device="cuda:0")
        sh.atomic_fetch_add(0, base + 64, 2**64 - 3, 1, res[0:])
        sh.atomic_fetch_add(2, base + 64, 5, 1, res[1:])
        sh.atomic_compare_swap(3, base + 72, 0, 9, 1, res[2:])
        sh.atomic_compare_swap(3, base + 72, 0, 11, 1, res[3:])
        sh.atomic_compare_swap(0, base + 72, 9, 11, 1, res[4:])
        sh.atomic_fetch_or(1, base + 80, 5, 3, res[5:])
        sh.atomic_fetch_or(1, base + 80, 6, 3, None)
        sh.stream_sync()
        exp = [w.atomic_fetch_add(0, 64, 2**64 - 3, 1), w.atomic_fetch_add(2, 64, 5, 1),
               w.atomic_compare_swap(3, 72, 0, 9, 1), w.atomic_compare_swap(3, 72, 0, 11, 1),
               w.atomic_compare_swap(0, 72, 9, 11, 1), w.atomic_fetch_or(1, 80, 5, 3)]
        w.atomic_fetch_or(1, 80, 6, 3)
        assert [int(x) for x in as_np(res, np.uint64)[:6]] == exp
        assert np.array_equal(heaps_of(heap, npes), w.heaps())


# ------------------------------------------------------------------ hash
# slot counts that are multiples of 8 take the sector-wide lookup, the others the slot-by-slot one; the
# shapes cover long chains over many sectors (load 0.8), wrap-around inside a single sector, and full tables
@pytest.mark.parametrize("npes,slots,n", [(16, 1 << 12, 30000), (5, 3001, 7000), (16, 64, 1200), (2, 1 << 12, 5800),
                                          (3, 8, 40), (4, 24, 60), (3, 8, 12)])
def test_hash_insert_lookup(npes, slots, n):
    keys = workgen.cfg4_keys(n=n)
    keys = np.concatenate([keys, keys[: n // 8]])        # duplicates; the last shape overfills
    queries = workgen.cfg4_queries(keys, n=2 * n + 3)
    hb = ((slots * 8 + 255) // 256 + 2) * 256
    w = oracle.World(npes, hb, oracle.SHUFFLED, 0)
    tab = w.malloc(slots * 8)
    ost = w.hash_insert(tab, slots, keys)
    ofound = w.hash_lookup(tab, slots, queries)
    otab = np.stack([w.heap(p)[tab:tab + 8 * slots].view(np.uint64) for p in range(npes)])
    with shmem_world(npes, hb) as (heap, base):
        t = sh.malloc(slots * 8)
        assert t - base == tab
        dk, dq = to_dev(keys), to_dev(queries)
        dst = torch.full((len(keys),), 255, dtype=torch.uint8, device="cuda:0")
        dfo = torch.full((len(queries),), 255, dtype=torch.uint8, device="cuda:0")
        sh.hash_insert(t, slots, dk, len(keys), dst, 3)
        sh.hash_lookup(t, slots, dq, len(queries), dfo, 2)
        sh.stream_sync()
        gtab = counters_of(heap, npes, tab, slots)
        st, found = as_np(dst, np.uint8), as_np(dfo, np.uint8)
    full = (ost == oracle.HASH_FULL).any()
    if not full:
        assert np.array_equal(gtab != 0, otab != 0)      # occupancy does not depend on the order
        for p in range(npes):
            assert np.array_equal(np.sort(gtab[p]), np.sort(otab[p]))
        assert np.array_equal(found, ofound)
        for code in (0, 1, 2):
            assert int((st == code).sum()) == int((ost == code).sum())
        # per key value: inserted exactly once, every other copy reported as duplicate
        order = np.argsort(keys, kind="stable")
        ks, ss = keys[order], st[order]
        firsts = np.r_[True, ks[1:] != ks[:-1]]
        ins_per_key = np.add.reduceat((ss == 0).astype(np.int64), np.flatnonzero(firsts))
        assert (ins_per_key == 1).all()
    else:
        # an overfull table: which keys fit depends on the order; check validity instead
        stored = gtab[gtab != 0]
        assert len(stored) == len(set(stored.tolist()))
        inserted = set(keys[st == 0].tolist())
        assert set(stored.tolist()) == inserted
        assert (st == 2).any()
        truth = np.array([int(q) in inserted for q in queries])
        assert np.array_equal(found.astype(bool), truth)
    # every stored key is reachable from its home slot before an empty one
    for p in range(npes):
        for s in np.flatnonzero(gtab[p])[:400]:
            h = oracle.mix64(int(gtab[p, s]))
            assert h % npes == p
            j = (h // npes) % slots
            while j != s:
                assert gtab[p, j] != 0
                j = (j + 1) % slots


def test_hash_table_not_sector_aligned():
    # a table that starts 8 bytes into an allocation: its groups of 8 slots straddle 64-byte sectors,
    # so the lookup takes the slot-by-slot kernel although the slot count is a multiple of 8
    npes, slots, n = 3, 512, 700
    keys = workgen.cfg4_keys(n=n)
    queries = workgen.cfg4_queries(keys, n=2 * n)
    hb = 1 << 14
    w = oracle.World(npes, hb, oracle.SHUFFLED, 0)
    tab = w.malloc(slots * 8 + 8) + 8
    ost = w.hash_insert(tab, slots, keys)
    ofound = w.hash_lookup(tab, slots, queries)
    with shmem_world(npes, hb) as (heap, base):
        t = sh.malloc(slots * 8 + 8) + 8
        assert t - base == tab
        dst = torch.full((n,), 255, dtype=torch.uint8, device="cuda:0")
        dfo = torch.full((2 * n,), 255, dtype=torch.uint8, device="cuda:0")
        sh.hash_insert(t, slots, to_dev(keys), n, dst, 2)
        sh.hash_lookup(t, slots, to_dev(queries), 2 * n, dfo, 2)
        sh.stream_sync()
        assert np.array_equal(as_np(dfo, np.uint8), ofound)
        assert np.array_equal(np.sort(as_np(dst, np.uint8)), np.sort(ost))


# ------------------------------------------------------------------ BFS
def check_tree(row, nbr, root, level, parent):
    reached = level >= 0
    assert parent[root] == root
    assert ((parent == sh.BFS_NONE) == ~reached).all()
    vs = np.flatnonzero(reached)
    vs = vs[vs != root]
    us = parent[vs].astype(np.int64)
    assert (level[us] == level[vs] - 1).all()
    for v, u in zip(vs[:3000], us[:3000]):                # the tree edge exists
        assert v in nbr[row[u]:row[u + 1]]


def run_bfs_case(row, nbr, roots, npes, wgs, mode=0):
    n = len(row) - 1
    vpp = -(-n // npes)
    hb = ((vpp * 28 + vpp // 8 + 16 * 256 + 255) // 256) * 256
    w = oracle.World(npes, hb, oracle.SHUFFLED, 1)
    with shmem_world(npes, hb) as (heap, base):
        drow, dnbr = to_dev(row), to_dev(nbr)
        g = sh.bfs_create(n, drow, dnbr, wgs)
        sh.bfs_configure(g, mode)
        dl = torch.empty(n, dtype=torch.int32, device="cuda:0")
        dp = torch.empty(n, dtype=torch.int32, device="cuda:0")
        for root in roots:
            stats = sh.bfs(g, int(root), dl, dp)
            sh.stream_sync()
            level, parent = as_np(dl, np.int32).copy(), as_np(dp, np.uint32).copy()
            olevel, oparent, ostats = w.bfs(row, nbr, int(root))
            assert np.array_equal(level, olevel)          # levels are unique
            ostats = dict(ostats, frontier_size=ostats["frontier_size"][:64])   # the C struct holds the first 64 levels
            assert stats == ostats                        # sizes per level, reached, traversed edges
            check_tree(row, nbr, int(root), level, parent)
            if mode & sh.BFS_CANONICAL_PARENTS:           # the one tree that can be compared vertex by vertex
                assert np.array_equal(parent, oracle.canonical_parents(row, nbr, olevel, int(root)))
        sh.bfs_destroy(g)
        assert sh.malloc(hb) == base                      # everything was returned to the heap


@pytest.mark.parametrize("mode", [sh.BFS_TOP_DOWN, sh.BFS_DIRECTION_OPTIMIZING, sh.BFS_BOTTOM_UP,
                                  sh.BFS_TOP_DOWN | sh.BFS_CANONICAL_PARENTS,
                                  sh.BFS_DIRECTION_OPTIMIZING | sh.BFS_CANONICAL_PARENTS])
@pytest.mark.parametrize("scale,npes,wgs", [(10, 16, 1), (14, 16, 4), (13, 3, 2), (16, 16, 8)])
def test_bfs_rmat(scale, npes, wgs, mode):
    row, nbr = workgen.rmat_csr(scale)
    roots = workgen.bfs_roots(row, 3)
    run_bfs_case(row, nbr, roots, npes, wgs, mode)


@pytest.mark.parametrize("mode", [sh.BFS_TOP_DOWN, sh.BFS_TOP_DOWN | sh.BFS_CANONICAL_PARENTS, sh.BFS_DIRECTION_OPTIMIZING])
@pytest.mark.parametrize("sort_div", ["0", "4000000000"])
def test_bfs_frontier_order(sort_div, mode, monkeypatch):
    # large frontiers are expanded from a queue rewritten in vertex order: never (0), or from 1024 vertices on
    # (a divisor beyond the vertex count leaves the floor); levels, statistics and the canonical tree do not
    # depend on the order
    monkeypatch.setenv("MI_SHMEM_BFS_SORT_DIV", sort_div)          # read by shmem_init
    for scale, npes, wgs in ((14, 16, 4), (16, 5, 8)):
        row, nbr = workgen.rmat_csr(scale)
        run_bfs_case(row, nbr, workgen.bfs_roots(row, 2), npes, wgs, mode)


@pytest.mark.parametrize("mode", [sh.BFS_TOP_DOWN | sh.BFS_CANONICAL_PARENTS, sh.BFS_DIRECTION_OPTIMIZING])
def test_bfs_rows_left_unsorted(mode, monkeypatch):
    # the library sorts the rows of its copy of the adjacency by the neighbours' degree rank; without that (the
    # path it also takes when the sort's memory cannot be had) the rows are only grouped by rank: same results
    monkeypatch.setenv("MI_SHMEM_BFS_SORT_ROWS", "0")             # read by shmem_init
    for scale, npes, wgs in ((13, 16, 4), (15, 3, 8)):
        row, nbr = workgen.rmat_csr(scale)
        run_bfs_case(row, nbr, workgen.bfs_roots(row, 2), npes, wgs, mode)


@pytest.mark.parametrize("mode", [sh.BFS_TOP_DOWN, sh.BFS_DIRECTION_OPTIMIZING, sh.BFS_BOTTOM_UP | sh.BFS_CANONICAL_PARENTS])
def test_bfs_deep_graphs(mode):
    # far more levels than the 64 whose sizes the statistics record: a path of 700 vertices with a few chords
    # and side branches, searched from one end, from the middle and from a leaf
    n = 900
    src = np.r_[np.arange(0, 699), [100, 250, 400, 400], np.arange(700, 760)].astype(np.uint32)
    dst = np.r_[np.arange(1, 700), [103, 252, 700, 760], np.arange(701, 761)].astype(np.uint32)
    row, nbr = workgen.csr_from_edges(n, src, dst)
    run_bfs_case(row, nbr, [0, 350, 699, 759], 3, 2, mode)


@pytest.mark.parametrize("mode", [sh.BFS_TOP_DOWN, sh.BFS_DIRECTION_OPTIMIZING | sh.BFS_CANONICAL_PARENTS, sh.BFS_BOTTOM_UP])
def test_bfs_searches_on_one_graph_do_not_see_each_other(mode):
    # two components (an R-MAT graph on the even vertex numbers and another on the odd ones) searched in turn
    # on one graph object: what a search leaves behind for the vertices of the other component (parent / level
    # records, bitmaps, queues) must not show in the next one, whose own component is all it may reach
    r1, n1 = workgen.rmat_csr(11)
    r2, n2 = workgen.rmat_csr(11, seed=77)
    na, nb = len(r1) - 1, len(r2) - 1
    src = np.r_[np.repeat(np.arange(na, dtype=np.uint32), np.diff(r1).astype(np.int64)) * 2,
                np.repeat(np.arange(nb, dtype=np.uint32), np.diff(r2).astype(np.int64)) * 2 + 1].astype(np.uint32)
    dst = np.r_[n1.astype(np.uint32) * 2, n2.astype(np.uint32) * 2 + 1].astype(np.uint32)
    keep = src < dst                                   # every undirected edge once; csr_from_edges stores both directions
    row, nbr = workgen.csr_from_edges(2 * max(na, nb), src[keep], dst[keep])
    deg = np.diff(row)
    even = [int(v) for v in np.flatnonzero(deg > 0) if v % 2 == 0]
    odd = [int(v) for v in np.flatnonzero(deg > 0) if v % 2 == 1]
    run_bfs_case(row, nbr, [even[0], odd[0], even[len(even) // 2], odd[-1], even[0]], 5, 3, mode)


@pytest.mark.parametrize("mode", [sh.BFS_TOP_DOWN, sh.BFS_DIRECTION_OPTIMIZING, sh.BFS_BOTTOM_UP])
def test_bfs_tiny_and_hub_graphs(mode):
    # a path, an isolated pair, and a star whose centre has more neighbours than
    # the long-row threshold (exercises the team-wide expansion)
    hub_deg = 5000
    src = np.r_[np.arange(0, 9), [20], np.full(hub_deg, 30)].astype(np.uint32)
    dst = np.r_[np.arange(1, 10), [21], np.arange(31, 31 + hub_deg)].astype(np.uint32)
    n = 31 + hub_deg + 5
    row, nbr = workgen.csr_from_edges(n, src, dst)
    run_bfs_case(row, nbr, [0, 9, 20, 30, 31, 4000, n - 1], 4, 2, mode)

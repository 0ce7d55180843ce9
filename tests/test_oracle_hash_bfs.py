"""Pins for the oracle's hash table and BFS, and sanity of the generators."""
import itertools

import numpy as np
import pytest
import scipy.sparse as sp
from scipy.sparse.csgraph import shortest_path

import oracle
import workgen

M64 = 2**64 - 1


def test_mixer_matches_published_splitmix64_outputs(golden_dir):
    vals = [int(l, 16) for l in open(f"{golden_dir}/splitmix64_seed0.txt")
            if l.strip() and not l.startswith("#")]
    assert len(vals) == 3
    for k, v in enumerate(vals, 1):
        assert oracle.mix64((k * 0x9E3779B97F4A7C15) & M64) == v


def py_home(key, npes, slots):
    h = oracle.mix64(key)
    return h % npes, (h // npes) % slots


def tables(w, off, slots):
    return np.stack([w.heap(p)[off:off + 8 * slots].view(np.uint64) for p in range(w.npes)])


@pytest.mark.parametrize("npes,slots,n", [(4, 64, 120), (16, 1024, 8000), (3, 80, 140)])
def test_hash_insert_lookup_membership_and_reachability(npes, slots, n):
    keys = workgen.cfg4_keys(n=n)
    keys = np.concatenate([keys, keys[: n // 10]])          # some duplicates
    w = oracle.World(npes, 256 * (-(-(slots * 8) // 256) + 16), oracle.SHUFFLED, 0)
    tab = w.malloc(slots * 8)
    st = w.hash_insert(tab, slots, keys)
    t = tables(w, tab, slots)
    stored = t[t != 0]
    assert len(stored) == len(set(stored.tolist()))          # no key stored twice
    truth = set(keys.tolist())
    assert set(stored.tolist()) == truth
    assert int((st == oracle.HASH_INSERTED).sum()) == len(truth)
    assert int((st == oracle.HASH_DUPLICATE).sum()) == len(keys) - len(truth)
    # each stored key sits in its owner's table, reachable from home before an EMPTY
    for p in range(npes):
        for s in np.flatnonzero(t[p]):
            o, home = py_home(int(t[p, s]), npes, slots)
            assert o == p
            j = home
            while j != s:
                assert t[p, j] != 0
                j = (j + 1) % slots
    q = workgen.cfg4_queries(keys, n=2 * n)
    found = w.hash_lookup(tab, slots, q)
    assert np.array_equal(found.astype(bool), np.array([int(x) in truth for x in q]))
    assert 0.3 < found.mean() < 0.7
    assert w.live_blocks() == 1                               # landing word was freed


def test_hash_full_and_duplicate_status():
    w = oracle.World(1, 4096, oracle.SHUFFLED, 0)
    keys = np.arange(1, 10, dtype=np.uint64)
    st = w.hash_insert(0, 8, keys)
    assert list(st[:8]) == [0] * 8 and st[8] == oracle.HASH_FULL
    assert list(w.hash_insert(0, 8, keys[:3])) == [1, 1, 1]
    assert list(w.hash_lookup(0, 8, np.array([1, 8, 9, 77], dtype=np.uint64))) == [1, 1, 0, 0]


def test_linear_probing_occupancy_is_order_independent():
    # the set of occupied slots does not depend on insertion order: all
    # permutations of a small key set over tiny tables
    rng = np.random.default_rng(5)
    for trial in range(6):
        npes, slots = int(rng.integers(1, 3)), int(rng.integers(4, 7))
        keys = rng.integers(1, 2**63, size=6, dtype=np.uint64)
        occ = None
        for perm in itertools.permutations(range(len(keys))):
            w = oracle.World(npes, 4096, oracle.SHUFFLED, 0)
            w.hash_insert(0, slots, keys[list(perm)])
            o = tables(w, 0, slots) != 0
            w.close()
            if occ is None:
                occ = o
            assert np.array_equal(o, occ)


# ------------------------------------------------------------------ BFS
def csr_to_scipy(row, nbr):
    n = len(row) - 1
    return sp.csr_matrix((np.ones(len(nbr), dtype=np.int8), nbr.astype(np.int64), row.astype(np.int64)),
                         shape=(n, n))


def check_bfs(row, nbr, root, level, parent, stats):
    n = len(row) - 1
    d = shortest_path(csr_to_scipy(row, nbr), method="D", unweighted=True, indices=int(root))
    exp = np.where(np.isinf(d), -1, d).astype(np.int32)
    assert np.array_equal(level, exp)                        # levels = shortest-path distances
    reached = level >= 0
    assert parent[root] == root
    assert ((parent == oracle.BFS_NONE) == ~reached).all()
    for v in np.flatnonzero(reached):
        if v == root:
            continue
        u = int(parent[v])
        assert level[u] == level[v] - 1
        assert v in nbr[row[u]:row[u + 1]]                   # the tree edge exists
    assert stats["reached"] == int(reached.sum())
    deg = np.diff(row).astype(np.int64)
    assert stats["edges_traversed"] == int(deg[reached].sum()) // 2
    assert stats["frontier_size"] == [int((level == l).sum()) for l in range(min(stats["nlevels"], 64))]   # the record holds 64 levels
    assert stats["nlevels"] == int(level.max()) + 1


def world_for(n, npes):
    vpp = -(-n // npes)
    hb = ((vpp * 16 + vpp // 8 + 8 * 256 + 255) // 256) * 256
    return oracle.World(npes, hb, oracle.SHUFFLED, 4)


@pytest.mark.parametrize("npes", [1, 3, 16])
def test_bfs_tiny_graphs(npes):
    # path 0-1-2-...-9, a star, an isolated pair, duplicate edges and a self-loop
    src = np.array([0, 1, 2, 3, 4, 5, 6, 7, 8, 10, 10, 10, 10, 15, 15, 3, 3, 20], dtype=np.uint32)
    dst = np.array([1, 2, 3, 4, 5, 6, 7, 8, 9, 11, 12, 13, 14, 16, 16, 4, 3, 21], dtype=np.uint32)
    n = 24
    row, nbr = workgen.csr_from_edges(n, src, dst)
    assert len(nbr) == 2 * (len(src) - 1)                    # self-loop dropped, duplicates kept
    for root in (0, 5, 9, 10, 13, 15, 20):
        w = world_for(n, npes)
        level, parent, stats = w.bfs(row, nbr, root)
        check_bfs(row, nbr, root, level, parent, stats)
        assert w.live_blocks() == 0
    w = world_for(n, npes)
    level, parent, stats = w.bfs(row, nbr, 0)
    assert list(level[:10]) == list(range(10)) and stats["nlevels"] == 10
    assert list(parent[1:10]) == list(range(9))


@pytest.mark.parametrize("npes", [1, 4])
def test_bfs_deep_path_and_cycle(npes):
    # closed forms far beyond the 64 levels whose sizes the record holds: on a path the level of a vertex is
    # its distance along the path, on a cycle the shorter way round
    n = 501
    row, nbr = workgen.csr_from_edges(n, np.arange(0, n - 1, dtype=np.uint32), np.arange(1, n, dtype=np.uint32))
    for root in (0, 137, n - 1):
        level, parent, stats = world_for(n, npes).bfs(row, nbr, root)
        assert np.array_equal(level, np.abs(np.arange(n) - root))
        assert stats["nlevels"] == max(root, n - 1 - root) + 1 and stats["reached"] == n and stats["edges_traversed"] == n - 1
        assert len(stats["frontier_size"]) == 64
        assert stats["frontier_size"] == [1] + [(1 if k <= root else 0) + (1 if k <= n - 1 - root else 0) for k in range(1, 64)]
        check_bfs(row, nbr, root, level, parent, stats)
    row, nbr = workgen.csr_from_edges(n, np.arange(0, n, dtype=np.uint32), (np.arange(0, n, dtype=np.uint32) + 1) % n)
    level, parent, stats = world_for(n, npes).bfs(row, nbr, 17)
    d = np.abs(np.arange(n) - 17)
    assert np.array_equal(level, np.minimum(d, n - d))
    assert stats["nlevels"] == n // 2 + 1 and stats["frontier_size"] == [1] + [2] * 63


@pytest.mark.parametrize("scale,npes", [(8, 4), (12, 16), (11, 5)])
def test_bfs_rmat_levels_are_shortest_paths(scale, npes):
    row, nbr = workgen.rmat_csr(scale)
    roots = workgen.bfs_roots(row, 4)
    for root in roots:
        w = world_for(1 << scale, npes)
        level, parent, stats = w.bfs(row, nbr, int(root))
        check_bfs(row, nbr, int(root), level, parent, stats)
        # a different delivery order gives the same levels (parents may differ)
        w2 = oracle.World(npes, w.heap_bytes, oracle.EAGER, 0)
        l2, p2, s2 = w2.bfs(row, nbr, int(root))
        assert np.array_equal(l2, level) and s2 == stats


# ------------------------------------------------------------------ generators
def test_rmat_generator_sanity():
    scale, ef = 12, 16
    src, dst = workgen.rmat_edges(scale, ef)
    assert len(src) == ef << scale and src.max() < (1 << scale) and dst.max() < (1 << scale)
    s2, d2 = workgen.rmat_edges(scale, ef)
    assert np.array_equal(src, s2) and np.array_equal(dst, d2)   # seeded
    row, nbr = workgen.csr_from_edges(1 << scale, src, dst)
    keep = src != dst
    assert row[-1] == 2 * int(keep.sum()) == len(nbr)
    a = csr_to_scipy(row, nbr)
    assert (a != a.T).nnz == 0                                   # symmetric, with multiplicity
    deg = np.diff(row)
    assert deg.max() > 20 * deg.mean()                           # skewed degrees
    # neighbour order = stable by edge position
    v = int(np.argmax(deg))
    exp = []
    for s, d in zip(src, dst):
        if s == d:
            continue
        if s == v:
            exp.append(d)
        if d == v:
            exp.append(s)
    assert np.array_equal(nbr[row[v]:row[v + 1]], np.array(exp, dtype=np.uint32))


def test_rmat_quadrant_frequencies():
    # raw labels (no relabelling): at every bit level the (row bit, column bit)
    # pair follows (a, b, c, d) = (0.57, 0.19, 0.19, 0.05)
    scale = 10
    src, dst = workgen.rmat_edges(scale, 64, relabel=False)
    for l in range(scale):
        r, c = (src >> l) & 1, (dst >> l) & 1
        freq = np.bincount((2 * r + c).astype(np.int64), minlength=4) / len(src)
        assert np.allclose(freq, [0.57, 0.19, 0.19, 0.05], atol=0.01), (l, freq)
    s2, d2 = workgen.rmat_edges(scale, 64, relabel=True)
    assert sorted(np.bincount(src, minlength=1 << scale)) == sorted(np.bincount(s2, minlength=1 << scale))
    s3, _ = workgen.rmat_edges(scale, 64, seed=2)
    assert not np.array_equal(s2, s3)


def test_zipf_and_amo_generators():
    rng = workgen.rng_for(1)
    idx = workgen.zipf_indices(rng, 200000, 1024)
    cnt = np.bincount(idx, minlength=1024).astype(float)
    assert idx.max() < 1024 and cnt[0] > cnt[1] > cnt[3] > cnt[15]
    assert abs(cnt[0] / cnt[1] - 2.0) < 0.15 and abs(cnt[0] / cnt[9] - 10.0) < 1.5
    pe, ix, a = workgen.cfg3_amo_ops(n=10000, npes=64, T=1)
    assert pe.min() >= 0 and pe.max() == 63 and (ix == 0).all() and (a == 1).all()
    keys = workgen.cfg4_keys(n=1000)
    assert keys.dtype == np.uint64 and keys.min() >= 1


def test_canonical_parents_against_loops():
    # the numpy form against the definition written as loops, on small R-MAT graphs
    for scale, seed in ((6, 1), (8, 2), (9, 3)):
        row, nbr = workgen.rmat_csr(scale, edge_factor=4, seed=seed)
        n = len(row) - 1
        root = int(workgen.bfs_roots(row, 1, seed=seed)[0])
        w = oracle.World(4, ((n // 4 + 1) * 40 + 8192 + 255) // 256 * 256, oracle.EAGER, 1)
        level, parent, _ = w.bfs(row, nbr, root)
        got = oracle.canonical_parents(row, nbr, level, root)
        for v in range(n):
            if v == root:
                assert got[v] == root
                continue
            want = oracle.BFS_NONE
            if level[v] > 0:
                for u in nbr[int(row[v]):int(row[v + 1])]:
                    if level[u] == level[v] - 1:
                        want = min(want, int(u))
            assert got[v] == want, (scale, v)
            if level[v] > 0:                    # and it is a valid tree edge, like the first-claimer parent
                assert level[parent[v]] == level[v] - 1 and level[got[v]] == level[v] - 1


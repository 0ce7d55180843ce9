"""Shapes nobody chose: the parity checks of the other GPU test files on sizes, PE counts, team sizes, table
loads, graph families and search modes drawn at random inside the documented limits.  A handful of seeds per
family by default; MI_SHMEM_RANDOM_CASES=<n> widens every family to n seeds (a few thousand take minutes)."""
import os

import numpy as np
import pytest

import workgen

pytestmark = pytest.mark.gpu

sh = pytest.importorskip("paper_2511_15076_amd")
import test_gpu_amo_hash_bfs as t_ahb  # noqa: E402
import test_gpu_moe as t_moe  # noqa: E402
import test_gpu_putget as t_pg  # noqa: E402
import test_gpu_sync as t_sync  # noqa: E402
import test_gpu_transpose as t_tr  # noqa: E402

SEEDS = range(100, 100 + int(os.environ.get("MI_SHMEM_RANDOM_CASES", "5")))
MODES = [sh.BFS_TOP_DOWN, sh.BFS_DIRECTION_OPTIMIZING, sh.BFS_BOTTOM_UP, sh.BFS_TOP_DOWN | sh.BFS_CANONICAL_PARENTS,
         sh.BFS_DIRECTION_OPTIMIZING | sh.BFS_CANONICAL_PARENTS, sh.BFS_BOTTOM_UP | sh.BFS_CANONICAL_PARENTS]


@pytest.mark.parametrize("seed", SEEDS)
def test_tables(seed):
    t_pg.test_random_mixed_tables_match_oracle(seed)


@pytest.mark.parametrize("seed", SEEDS)
def test_moe_small(seed):
    t_moe.test_dispatch_and_combine_match_oracle(*t_moe._random_case(seed))


@pytest.mark.parametrize("seed", SEEDS)
def test_moe_large(seed):
    rng = np.random.default_rng(17000 + seed)
    P = int(rng.choice([2, 4, 8, 16]))
    epp = int(rng.choice([1, 2, 4, 9, 36]))
    T = int(rng.integers(1, 129))
    K = int(rng.integers(1, min(P * epp, 8) + 1))
    Hb = 16 * int(rng.integers(1, 900))
    while P * epp * P * T * Hb > (192 << 20):           # the receive buffers of all PEs, kept to what the oracle does in a blink
        Hb = max(16, Hb // 32 * 16)
        if Hb == 16:
            T = max(1, T // 2)
    ntok = [int(rng.integers(0, T + 1)) for _ in range(P)]
    wgs = min(256 // P, int(rng.choice([1, 5, 8, 16, 32, 36, 64])))      # the teams of a launch must be co-resident
    t_moe.test_dispatch_and_combine_match_oracle(P, P * epp, T, K, Hb, ntok, str(rng.choice(["uniform", "zipf"])),
                                                 float(rng.choice([0.0, 0.0, 0.25])), wgs)


def _hash_case(monkeypatch, seed, npes, slots, load, wgs_insert, wgs_lookup):
    n = max(8, int(npes * slots * load / 1.125))         # the test body adds n / 8 duplicates
    keys0, queries0, insert0, lookup0 = workgen.cfg4_keys, workgen.cfg4_queries, sh.hash_insert, sh.hash_lookup
    monkeypatch.setattr(workgen, "cfg4_keys", lambda n: keys0(seed=5000 + seed, n=n))
    monkeypatch.setattr(workgen, "cfg4_queries", lambda keys, n: queries0(keys, seed=6000 + seed, n=n))
    monkeypatch.setattr(sh, "hash_insert", lambda t, s, k, m, out, w: insert0(t, s, k, m, out, wgs_insert))
    monkeypatch.setattr(sh, "hash_lookup", lambda t, s, k, m, out, w: lookup0(t, s, k, m, out, wgs_lookup))
    t_ahb.test_hash_insert_lookup(npes, slots, n)


@pytest.mark.parametrize("seed", SEEDS)
def test_hash_small(monkeypatch, seed):
    rng = np.random.default_rng(9000 + seed)
    npes = int(rng.integers(1, 17))
    slots = int(rng.integers(1, 600)) * 8 if rng.random() < 0.6 else int(rng.integers(1, 5000))
    load = float(rng.choice([0.05, 0.3, 0.5, 0.8, 0.95, 1.1]))                # the last overfills the table
    _hash_case(monkeypatch, seed, npes, slots, load, int(rng.integers(1, 5)), int(rng.integers(1, 5)))


@pytest.mark.parametrize("seed", SEEDS)
def test_hash_large(monkeypatch, seed):
    rng = np.random.default_rng(19000 + seed)
    npes = int(rng.choice([1, 8, 16, 64]))
    slots = int(rng.integers(1 << 9, 1 << 16)) // 8 * 8 + (0 if rng.random() < 0.7 else int(rng.integers(1, 8)))
    load = float(rng.choice([0.3, 0.5, 0.8, 0.95]))
    cap = 64 if npes == 64 else 256
    _hash_case(monkeypatch, seed, npes, slots, load, min(cap, int(rng.choice([1, 4, 16, 64, 256]))),
               min(cap, int(rng.choice([1, 4, 16, 64, 256]))))


def _graph(rng, seed, large):
    kind = 0 if large else int(rng.integers(0, 3))
    if kind == 0:                                        # R-MAT of several skews and densities
        scale = int(rng.integers(15, 20)) if large else int(rng.integers(6, 16))
        ef = int(rng.choice([4, 16, 32] if large else [1, 4, 16, 40]))
        a = float(rng.choice([0.45, 0.57, 0.65] if large else [0.25, 0.45, 0.57, 0.7]))
        return workgen.rmat_csr(scale, ef, (a, (1 - a) / 3, (1 - a) / 3), seed=777 + seed)
    if kind == 1:                                        # uniform random, from far below to far above the giant-component threshold
        n = int(rng.integers(2, 40000))
        m = int(n * float(rng.choice([0.5, 1.0, 3.0, 10.0])))
        return workgen.csr_from_edges(n, rng.integers(0, n, m).astype(np.uint32), rng.integers(0, n, m).astype(np.uint32))
    n = int(rng.integers(3000, 30000))                   # a few rows beyond the long-row threshold, a sparse background, a path
    src = [rng.integers(0, n, n // 2), np.arange(0, 500)]
    dst = [rng.integers(0, n, n // 2), np.arange(1, 501)]
    for h in rng.integers(0, n, int(rng.integers(1, 5))):
        d = int(rng.integers(900, 6000))
        src.append(np.full(d, h))
        dst.append(rng.integers(0, n, d))
    return workgen.csr_from_edges(n, np.concatenate(src).astype(np.uint32), np.concatenate(dst).astype(np.uint32))


def _bfs_case(seed, large):
    rng = np.random.default_rng((21000 if large else 11000) + seed)
    npes = int(rng.choice([1, 3, 8, 16])) if large else int(rng.integers(1, 17))
    wgs = int(rng.choice([8, 16, 32, 64])) if large else int(rng.integers(1, 9))
    mode = MODES[int(rng.integers(0, len(MODES)))]
    row, nbr = _graph(rng, seed, large)
    deg = np.diff(row)
    if int((deg > 0).sum()) < 3:
        pytest.skip("a graph with hardly an edge")
    roots = list(workgen.bfs_roots(row, 2, seed=seed)) + [int(np.argmax(deg))]
    t_ahb.run_bfs_case(row, nbr, roots, npes, wgs, mode)


@pytest.mark.parametrize("seed", SEEDS)
def test_bfs_small(seed):
    _bfs_case(seed, False)


@pytest.mark.parametrize("seed", SEEDS)
def test_bfs_large(seed):
    _bfs_case(seed, True)


@pytest.mark.parametrize("seed", SEEDS)
def test_transpose(seed):
    rng = np.random.default_rng(13000 + seed)
    npes = int(rng.integers(1, 9))
    wgs = int(rng.integers(1, 9)) if rng.random() < 0.7 else 1024 // npes       # small teams, or a launch large enough for the wide tiles
    t_tr.test_transpose_matches_igets(npes, npes * int(rng.integers(1, 200)), int(rng.choice([4, 8])), wgs)


@pytest.mark.parametrize("seed", SEEDS)
def test_fetch_add(seed):
    rng = np.random.default_rng(15000 + seed)
    t_ahb.test_fetch_add_batch(int(rng.integers(0, 2)), str(rng.choice(["uniform", "zipf"])),
                               int(rng.choice([1, 2, 63, 64, 65, 1000, 4096])), int(rng.choice([1, 2, 3, 7, 16, 64])))


@pytest.mark.parametrize("seed", SEEDS)
def test_sweep_cell(seed):
    rng = np.random.default_rng(23000 + seed)
    kind = int(rng.integers(0, 4))
    if kind < workgen.OP_IPUT:
        # every vector width of the small-message path, the chunked path and its tails
        count = int(rng.choice([int(rng.integers(1, 64)), int(rng.integers(1, 129)) * 8, int(rng.integers(1, 5000)),
                                (1 << int(rng.integers(10, 21))) + int(rng.integers(0, 9)) * 8, int(rng.integers(1, 1 << 21))]))
        eb, rs, ls = 1, 1, 1
    else:
        count, eb = int(rng.integers(1, 6000)), int(rng.choice([1, 2, 4, 8]))
        rs, ls = int(rng.choice([1, 1, 2, 3, 16, 70])), int(rng.choice([1, 1, 2, 5, 32]))
    nops = int(rng.integers(1, 300)) if count * eb * max(rs, ls) < (1 << 16) else int(rng.integers(1, 6))
    nslots = int(rng.integers(1, nops + 1))
    t_pg.test_copy_sweep_cell((kind, count, eb, rs, ls, nops, nslots, int(rng.choice([1, 2, 3, 5, 8, 16, 32]))))


@pytest.mark.parametrize("seed", SEEDS)
def test_single_put_get_iput_iget(seed):
    # stand-alone operations, one after the other with a barrier between them (so overlapping ranges are
    # fine): any size from nothing to megabytes at any byte alignment, any pair of PEs, self included
    import torch
    from gpu_util import heaps_of, shmem_world
    rng = np.random.default_rng(25000 + seed)
    npes, hb = int(rng.integers(1, 5)), 12 << 20
    init = t_pg.seeded_heaps(npes, hb, 3000 + seed)
    w = t_pg.oracle_world(init)
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        for k in range(10):
            me, pe = int(rng.integers(0, npes)), int(rng.integers(0, npes))
            if rng.random() < 0.6:
                n = int(rng.choice([int(rng.integers(0, 300)), int(rng.integers(0, 70000)), int(rng.integers(1 << 20, 5 << 20)),
                                    (int(rng.integers(1, 5)) << 20) + 16 * int(rng.integers(0, 300))]))
                al = int(rng.choice([1, 8, 16, 256]))
                lo = int(rng.integers(0, (hb // 2 - n) // al + 1)) * al              # local range in the low half
                so = hb // 2 + int(rng.integers(0, (hb // 2 - n) // al + 1)) * al    # remote range in the high half
                if k % 2:
                    assert w.put(me, so, lo, n, pe) == 0
                    sh.put(me, base + so, sh.ptr(base + lo, me), n, pe)
                else:
                    assert w.get(me, lo, so, n, pe) == 0
                    sh.get(me, sh.ptr(base + lo, me), base + so, n, pe)
            else:
                eb = int(rng.choice([1, 2, 4, 8]))
                ds, ss = int(rng.choice([1, 2, 3, 7, 64])), int(rng.choice([1, 2, 5, 9, 33]))
                n = int(rng.integers(0, min(20000, (hb // 2 - 1024) // (max(ds, ss) * eb))))
                lo = int(rng.integers(0, 64)) * eb
                so = hb // 2 + int(rng.integers(0, 64)) * eb
                if k % 2:
                    assert w.iput(me, so, lo, ds, ss, n, eb, pe) == 0
                    sh.iput(me, base + so, sh.ptr(base + lo, me), ds, ss, n, eb, pe)
                else:
                    assert w.iget(me, lo, so, ds, ss, n, eb, pe) == 0
                    sh.iget(me, sh.ptr(base + lo, me), base + so, ds, ss, n, eb, pe)
            sh.barrier_all()
            w.barrier_all()
        assert np.array_equal(heaps_of(heap, npes), w.heaps())


@pytest.mark.parametrize("seed", SEEDS)
def test_ring_pingpong_barrier(seed):
    # persistent launches: every workgroup must be resident, so PEs x team stays within the 256 CUs
    rng = np.random.default_rng(27000 + seed)
    n = int(rng.choice([1, 2, 3, 5, 8, 16, 32]))
    ds = int(rng.choice([8 * int(rng.integers(1, 40)), 8 * int(rng.integers(1, 9000)), (1 << int(rng.integers(12, 20))) + 8 * int(rng.integers(0, 40))]))
    ds = min(ds, (128 << 20) // (n * n) // 8 * 8)        # all heaps together stay within 256 MiB
    t_sync.ring_cases([(n, ds)], int(rng.integers(1, max(1, min(8, 256 // n)) + 1)), int(rng.integers(1, 6)))
    t_sync.pingpong_case(int(rng.integers(2, 6)), int(rng.choice([8 * int(rng.integers(1, 64)), int(rng.integers(1, 70000))])),
                         int(rng.integers(1, 60)))
    npes = int(rng.choice([1, 2, 3, 7, 16, 64]))
    t_sync.test_barrier_epochs(npes, int(rng.integers(1, max(1, min(40, 256 // npes)) + 1)), int(rng.integers(1, 400)))


@pytest.mark.parametrize("seed", SEEDS)
def test_compare_swap(seed):
    rng = np.random.default_rng(29000 + seed)
    t_ahb.test_compare_swap_claim_batch(str(rng.choice(["uniform", "zipf"])), int(rng.choice([1, 2, 64, 100, 1024, 8192])))


@pytest.mark.parametrize("seed", SEEDS)
def test_tables_with_large_ops(seed):
    # tables that mix team-wide operations (above 64 KiB, up to 2 MiB, contiguous and strided, any alignment)
    # with small ones; every op of a window owns one local and one remote 2 MiB stripe
    import torch
    from gpu_util import heaps_of, shmem_world, to_dev
    rng = np.random.default_rng(31000 + seed)
    npes, stripes, sb = int(rng.integers(2, 5)), 5, 2 << 20
    hb = 2 * stripes * sb
    window = int(rng.integers(1, stripes + 1))
    nwin = 4
    ops = np.zeros(window * nwin, dtype=workgen.OP_DESC)
    for wdx in range(nwin):
        free_l = [list(rng.permutation(stripes)) for _ in range(npes)]
        free_r = [list(rng.permutation(stripes)) for _ in range(npes)]
        for k in range(window):
            me, pe = int(rng.integers(0, npes)), int(rng.integers(0, npes))
            lo = int(free_l[me].pop()) * sb
            so = (stripes + int(free_r[pe].pop())) * sb
            kind = int(rng.integers(0, 4))
            if kind < 2:
                n = int(rng.choice([int(rng.integers(0, 5000)), int(rng.integers(60000, 70000)), 65536, 65536 + 16,
                                    4096 * int(rng.integers(17, 400)), 16 * int(rng.integers(4097, 120000)),
                                    int(rng.integers(65537, sb - 8192))]))
                al = int(rng.choice([1, 8, 16, 4096]))
                a, b = int(rng.integers(0, 4096 // al)) * al, int(rng.integers(0, 4096 // al)) * al
                ops[wdx * window + k] = (kind, me, pe, 1, lo + a, so + b, n, 1, 1, 0)
            else:
                eb = int(rng.choice([1, 2, 4, 8]))
                ls, ss = int(rng.integers(1, 6)), int(rng.integers(1, 6))
                cnt = int(rng.integers(0, (sb // eb - 64) // max(ls, ss) + 1))
                a, b = int(rng.integers(0, 8)) * eb, int(rng.integers(0, 8)) * eb
                ops[wdx * window + k] = (kind, me, pe, eb, lo + a, so + b, cnt, ls, ss, 0)
    init = t_pg.seeded_heaps(npes, hb, 500 + seed)
    w = t_pg.oracle_world(init)
    assert w.op_batch(ops, window) == 0
    want = w.heaps()
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        sh.op_batch(to_dev(ops), len(ops), window, int(rng.choice([1, 4, 16, 33, 64])))
        sh.stream_sync()
        assert np.array_equal(heaps_of(heap, npes), want)


@pytest.mark.parametrize("seed", SEEDS)
def test_team_barriers(seed):
    # disjoint strided teams (one per residue class of the stride) at different paces in one launch
    import test_gpu_teams as t_teams
    rng = np.random.default_rng(33000 + seed)
    npes = int(rng.integers(1, 41))
    stride = int(rng.integers(1, 5))
    plan = []
    for r in range(min(stride, npes)):
        if rng.random() < 0.75:
            start = r + stride * int(rng.integers(0, 3))
            if start >= npes:
                continue
            size = int(rng.integers(1, (npes - 1 - start) // stride + 2))
            plan.append(((start, stride, size), int(rng.choice([0, 1, 2, 17, 150, 400]))))
    if not plan:
        plan = [((0, 1, npes), 25)]
    t_teams.test_team_epochs_match_oracle(npes, int(rng.integers(1, min(4, 256 // npes) + 1)), plan)

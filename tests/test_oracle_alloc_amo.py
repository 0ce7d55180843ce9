"""Pins for the oracle's symmetric allocator and its atomic memory operations."""
import itertools

import numpy as np
import pytest

import oracle
import workgen

G = 256


def test_allocator_against_bitmap_model():
    # independent model: a bitmap of 256-byte granules; first fit = lowest address
    rng = np.random.default_rng(7)
    for trial in range(20):
        hb = G * int(rng.integers(8, 64))
        w = oracle.World(3, hb, oracle.EAGER, 0)
        used = np.zeros(hb // G, dtype=bool)
        live = {}
        for step in range(300):
            if live and rng.random() < 0.45:
                off = list(live)[int(rng.integers(0, len(live)))]
                g = live.pop(off)
                assert w.free(off) == 0
                used[off // G: off // G + g] = False
            else:
                n = int(rng.integers(1, 6 * G))
                g = (n + G - 1) // G
                exp = -1
                for s in range(0, hb // G - g + 1):
                    if not used[s:s + g].any():
                        exp = s * G
                        break
                got = w.malloc(n)
                assert got == exp, (trial, step, n)
                if got >= 0:
                    assert got % G == 0
                    used[got // G: got // G + g] = True
                    live[got] = g
            assert w.live_blocks() == len(live)
        for off in list(live):
            assert w.free(off) == 0
        assert w.malloc(hb) == 0                      # everything coalesced again


def test_allocator_edge_cases():
    w = oracle.World(2, 16 * G, oracle.EAGER, 0)
    assert w.malloc(0) == -1
    assert w.align(3, 8) == -1                        # alignment must be a power of two
    a = w.malloc(1)
    b = w.align(1024, 10)
    assert a == 0 and b == 1024
    assert w.malloc(16 * G) == -1                     # exhaustion
    assert w.free(b + G) == -8 and w.free(12345) == -8 and w.free(-1) == -8
    assert w.free(a) == 0 and w.free(a) == -8         # double free
    c = w.malloc(G)
    assert c == a                                     # freed block is reused
    assert w.malloc(3 * G) == G                       # the hole below the aligned block


def test_fetch_add_wraps_and_returns_old():
    w = oracle.World(2, 4096, oracle.SHUFFLED, 0)
    assert w.atomic_fetch_add(0, 8, 2**64 - 3, 1) == 0
    assert w.atomic_fetch_add(1, 8, 5, 1) == 2**64 - 3
    assert w.atomic_fetch_add(0, 8, 0, 1) == 2        # wrapped mod 2^64
    assert int(w.heap(0)[8:16].view(np.uint64)[0]) == 0   # other PE's copy untouched
    with pytest.raises(RuntimeError):
        w.atomic_fetch_add(0, 4, 1, 1)                # misaligned
    with pytest.raises(RuntimeError):
        w.atomic_fetch_add(0, 4096, 1, 1)             # out of range


def test_compare_swap_and_fetch_or_definition():
    w = oracle.World(2, 4096, oracle.SHUFFLED, 0)
    assert w.atomic_compare_swap(0, 0, 0, 7, 1) == 0      # succeeded: saw cond
    assert w.atomic_compare_swap(0, 0, 0, 9, 1) == 7      # failed: value kept
    assert w.atomic_compare_swap(0, 0, 7, 9, 1) == 7
    assert int(w.heap(1)[0:8].view(np.uint64)[0]) == 9
    assert w.atomic_fetch_or(1, 16, 0b0101, 0) == 0
    assert w.atomic_fetch_or(1, 16, 0b0110, 0) == 0b0101
    assert int(w.heap(0)[16:24].view(np.uint64)[0]) == 0b0111


@pytest.mark.parametrize("dist,T", [("uniform", 1), ("uniform", 64), ("zipf", 64), ("zipf", 1024)])
def test_fetch_add_batch_is_a_permutation_of_prefix_sums(dist, T):
    npes, n = 8, 20000
    pe, idx, a = workgen.cfg3_amo_ops(n=n, npes=npes, T=T, dist=dist, addend="rand16")
    w = oracle.World(npes, max(4096, T * 8), oracle.SHUFFLED, 0)
    ctr = w.malloc(T * 8)
    old = w.amo_batch(oracle.AMO_FETCH_ADD, ctr, pe, idx, a)
    final = np.stack([w.heap(p)[ctr:ctr + 8 * T].view(np.uint64) for p in range(npes)])
    # closed form for the final counters
    exp = np.zeros((npes, T), dtype=np.uint64)
    np.add.at(exp, (pe, idx), a)
    assert np.array_equal(final, exp)
    # per counter: sorted by fetched value, f0 = 0 and f[k+1] = f[k] + a[k]
    key = pe.astype(np.int64) * T + idx
    order = np.lexsort((old, key))
    k, f, aa = key[order], old[order], a[order]
    first = np.r_[True, k[1:] != k[:-1]]
    assert (f[first] == 0).all()
    same = ~first[1:]
    assert np.array_equal(f[1:][same], (f[:-1] + aa[:-1])[same])


def test_fetch_add_one_fetches_0_to_n_minus_1():
    npes, n, T = 4, 5000, 3
    pe, idx, a = workgen.cfg3_amo_ops(n=n, npes=npes, T=T, addend="one")
    w = oracle.World(npes, 4096, oracle.SHUFFLED, 0)
    old = w.amo_batch(oracle.AMO_FETCH_ADD, 0, pe, idx, a)
    for p in range(npes):
        for t in range(T):
            m = (pe == p) & (idx == t)
            assert sorted(old[m]) == list(range(int(m.sum())))


def test_min_cas_loop_and_claim_closed_forms():
    npes, n, T = 4, 6000, 16
    pe, idx, tag = workgen.cfg3_amo_ops(n=n, npes=npes, T=T, dist="zipf", addend="tag")
    tag = np.random.default_rng(1).permutation(tag)   # so that the minimum is not always first
    w = oracle.World(npes, 4096, oracle.SHUFFLED, 0)
    w.amo_batch(oracle.AMO_MIN_CAS_LOOP, 0, pe, idx, tag)
    final = np.stack([w.heap(p)[0:8 * T].view(np.uint64) for p in range(npes)])
    exp = np.zeros((npes, T), dtype=np.uint64)
    for p, i, t in zip(pe, idx, tag):
        if exp[p, i] == 0 or t < exp[p, i]:
            exp[p, i] = t
    assert np.array_equal(final, exp)
    # single-shot claim: exactly one op per touched slot sees 0, the rest see the winner
    w2 = oracle.World(npes, 4096, oracle.SHUFFLED, 0)
    old = w2.amo_batch(oracle.AMO_COMPARE_SWAP, 0, pe, idx, np.zeros(n, np.uint64), tag)
    fin2 = np.stack([w2.heap(p)[0:8 * T].view(np.uint64) for p in range(npes)])
    key = pe.astype(np.int64) * T + idx
    for k in np.unique(key):
        m = key == k
        winners = np.flatnonzero(m & (old == 0))
        assert len(winners) == 1
        win = tag[winners[0]]
        assert fin2.reshape(-1)[k] == win
        assert (old[m & (old != 0)] == win).all()
    assert int((fin2 != 0).sum()) == len(np.unique(key))


# ---- brute force: every interleaving of atomic steps on tiny inputs -----------
def _interleavings(lens):
    """All orders of op slots that keep each issuer's program order."""
    seq = []
    for who, n in enumerate(lens):
        seq += [who] * n
    return set(itertools.permutations(seq))


def _run_schedule(progs, schedule, nslots):
    """Python definition of compare-and-swap executed in the given order."""
    mem = [0] * nslots
    pc = [0] * len(progs)
    seen = [[] for _ in progs]
    for who in schedule:
        slot, cond, val = progs[who][pc[who]]
        pc[who] += 1
        cur = mem[slot]
        if cur == cond:
            mem[slot] = val
        seen[who].append(cur)
    return tuple(mem), tuple(tuple(s) for s in seen)


def test_compare_swap_linearisable_by_brute_force():
    rng = np.random.default_rng(3)
    for trial in range(25):
        nissuers = int(rng.integers(2, 4))
        lens = [int(rng.integers(1, 4)) for _ in range(nissuers)]
        nslots = int(rng.integers(1, 3))
        progs = [[(int(rng.integers(0, nslots)), int(rng.integers(0, 3)), int(rng.integers(1, 4)))
                  for _ in range(l)] for l in lens]
        allowed = set()
        for sched in _interleavings(lens):
            allowed.add(_run_schedule(progs, sched, nslots))
            # the oracle, driven in this very order, must reproduce the model exactly
            w = oracle.World(nissuers, 4096, oracle.SHUFFLED, 0)
            pc = [0] * nissuers
            seen = [[] for _ in progs]
            for who in sched:
                slot, cond, val = progs[who][pc[who]]
                pc[who] += 1
                seen[who].append(w.atomic_compare_swap(who, 8 * slot, cond, val, 0))
            mem = tuple(int(x) for x in w.heap(0)[0:8 * nslots].view(np.uint64))
            assert (mem, tuple(tuple(s) for s in seen)) == _run_schedule(progs, sched, nslots)
            w.close()
        assert len(allowed) >= 1

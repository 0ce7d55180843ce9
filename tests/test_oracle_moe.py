"""Pins for the MoE-shaped dispatch/combine oracle (CPU only).

The oracle walks senders, experts and tokens with one-sided puts and signals.  It is held
against things it does not contain: a hand-worked routing example, a sort-based restatement of
"who receives what", closed forms of the combine sum, the paper's message sizes, and the
delivery-order independence that the signal ordering rule must give.
"""
import numpy as np
import pytest

import oracle
import workgen
from oracle import moe


def run_dispatch(npes, E, T, K, Hb, x, topk, ntok, mode=oracle.SHUFFLED, seed=3):
    lay = moe.MoeLayout(npes, E, T, K, Hb)
    w = oracle.World(npes, lay.end, mode, seed)
    for p in range(npes):
        w.heap(p)[:] = 0
    out = moe.dispatch(w, lay, x, topk, ntok)
    return w, lay, out


def expected_by_sorting(npes, E, T, K, topk, ntok):
    """Routes as one table sorted by (expert, sender, token): the packed order, restated."""
    s, t, j = np.nonzero(topk >= 0)
    keep = t < ntok[s]
    s, t, j = s[keep], t[keep], j[keep]
    e = topk[s, t, j]
    order = np.lexsort((t, s, e))
    return e[order], s[order], t[order], j[order]


def test_worked_example(golden_dir):
    cfg, routes, ntok, arrivals, ranges = {}, [], None, {}, {}
    for line in open(f"{golden_dir}/moe_dispatch_worked.txt"):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = line.split()
        if f[0] == "config":
            cfg = {k: int(v) for k, v in (kv.split("=") for kv in f[1:])}
        elif f[0] == "route":
            routes.append(tuple(map(int, f[1:])))
        elif f[0] == "ntok":
            ntok = np.array(f[1:], dtype=np.int32)
        elif f[0] == "expert":
            items = " ".join(f[3:]).split(";")
            arrivals[int(f[1])] = [tuple(map(int, it.split())) for it in items]
        elif f[0] == "range":
            ranges[(int(f[1]), int(f[2]))] = (int(f[3]), int(f[4]))
    P, E, T, K = cfg["npes"], cfg["experts"], cfg["max_tokens"], cfg["topk"]
    topk = np.full((P, T, K), -1, dtype=np.int32)
    for pe, t, a, b in routes:
        topk[pe, t] = (a, b)
    Hb = 8
    x = workgen.moe_tokens(5, P, T, Hb)
    _, lay, (rx, info, rng, cnt) = run_dispatch(P, E, T, K, Hb, x, topk, ntok)
    epp = E // P
    for e, items in arrivals.items():
        r, le = divmod(e, epp)
        assert cnt[r, le] == len(items)
        for i, (t, s, j) in enumerate(items):
            assert tuple(info[r, le, i]) == (t, s, j, e)
            assert np.array_equal(rx[r, le, i], x[s, t])
        assert not rx[r, le, len(items):].any()
    for (e, s), bc in ranges.items():
        r, le = divmod(e, epp)
        assert tuple(rng[r, le, s]) == bc


@pytest.mark.parametrize("P,E,T,K,Hb,dist,drop", [
    (4, 16, 8, 3, 32, "uniform", 0.0),
    (4, 8, 16, 4, 16, "zipf", 0.2),
    (3, 9, 5, 9, 8, "uniform", 0.0),      # every token goes to every expert
    (2, 2, 7, 1, 64, "uniform", 0.0),
])
@pytest.mark.parametrize("mode", [oracle.AT_QUIET, oracle.SHUFFLED])
def test_dispatch_matches_sorted_routes(P, E, T, K, Hb, dist, drop, mode):
    topk, ntok = workgen.moe_routing(11, P, E, T, K, ntok=[T, 0, T // 2, T][:P], dist=dist, drop=drop)
    x = workgen.moe_tokens(12, P, T, Hb)
    _, lay, (rx, info, rng, cnt) = run_dispatch(P, E, T, K, Hb, x, topk, ntok, mode)
    e, s, t, j = expected_by_sorting(P, E, T, K, topk, ntok)
    assert cnt.sum() == len(e)                                    # every route arrives exactly once
    epp = E // P
    pos = 0
    for ee in range(E):
        r, le = divmod(ee, epp)
        n = int((e == ee).sum())
        assert cnt[r, le] == n
        sl = slice(pos, pos + n)
        assert np.array_equal(info[r, le, :n], np.stack([t[sl], s[sl], j[sl], e[sl]], axis=1))
        assert np.array_equal(rx[r, le, :n], x[s[sl], t[sl]])
        per_sender = np.bincount(s[sl], minlength=P)
        assert np.array_equal(rng[r, le, :, 1], per_sender)
        assert np.array_equal(rng[r, le, :, 0], np.cumsum(per_sender) - per_sender)
        pos += n


def test_message_is_metadata_plus_token_at_paper_sizes():
    # hidden 7168 in 16-bit words = 14,336 bytes of token data; message = 14,352 bytes (Sec. V-C)
    P, E, T, K, Hb = 2, 2, 2, 1, 14336
    topk = np.array([[[1], [1]], [[-1], [-1]]], dtype=np.int32)     # PE 0 sends both tokens to expert 1
    ntok = np.array([2, 0], dtype=np.int32)
    x = workgen.moe_tokens(1, P, T, Hb)
    w, lay, _ = run_dispatch(P, E, T, K, Hb, x, topk, ntok)
    assert lay.msg == 14352
    h = w.heap(1)
    first = lay.slot(0, 0, 0)
    assert np.array_equal(h[first:first + 16].view(np.int32), [0, 0, 0, 1])
    assert np.array_equal(h[first + 14352:first + 14352 + 16].view(np.int32), [1, 0, 0, 1])   # next slot starts here
    assert np.array_equal(h[first + 16:first + 14352], x[0, 0])
    assert np.array_equal(h[first + 14352 + 16:first + 2 * 14352], x[0, 1])


def test_signals_carry_count_plus_one_and_are_reset():
    P, E, T, K, Hb = 2, 4, 4, 2, 8
    topk, ntok = workgen.moe_routing(3, P, E, T, K)
    x = workgen.moe_tokens(4, P, T, Hb)
    lay = moe.MoeLayout(P, E, T, K, Hb)
    w = oracle.World(P, lay.end, oracle.EAGER, 1)
    for p in range(P):
        w.heap(p)[:] = 0
    seen = {}
    real = w.signal_add

    def spy(pe_self, sym, value, pe):
        seen[(pe, sym)] = value
        return real(pe_self, sym, value, pe)
    w.signal_add = spy
    _, _, rng, _ = moe.dispatch(w, lay, x, topk, ntok)
    epp = E // P
    for r in range(P):
        for le in range(epp):
            for s in range(P):
                assert seen[(r, lay.dsig + 8 * (le * P + s))] == rng[r, le, s, 1] + 1
        assert not w.heap(r)[lay.dsig:lay.dsig + 8 * epp * P].any()


@pytest.mark.parametrize("mode", [oracle.AT_QUIET, oracle.SHUFFLED])
def test_combine_closed_forms(mode):
    P, E, T, K, Hb = 4, 12, 6, 3, 32
    topk, ntok = workgen.moe_routing(21, P, E, T, K, ntok=[6, 1, 0, 4], drop=0.25)
    x = workgen.moe_tokens(22, P, T, Hb)
    w, lay, (rx, info, rng, cnt) = run_dispatch(P, E, T, K, Hb, x, topk, ntok, mode)
    # identity experts: every valid route returns the token itself -> nvalid * x (mod 2^32)
    got = moe.combine(w, lay, rx, info, rng, topk, ntok, epoch=1)
    nvalid = (topk >= 0).sum(axis=2).astype(np.uint32)
    want = (x.view(np.uint32).reshape(P, T, Hb // 4) * nvalid[:, :, None]).astype(np.uint32)
    for p in range(P):
        want[p, ntok[p]:] = 0
    assert np.array_equal(got.view(np.uint32).reshape(P, T, Hb // 4), want)
    # experts that add (expert id + 1) to every word -> nvalid * x + sum of (e + 1)
    eo = rx.view(np.uint32).reshape(P, E // P, P * T, Hb // 4).copy()
    for r in range(P):
        for le in range(E // P):
            eo[r, le, :cnt[r, le]] += np.uint32(r * (E // P) + le + 1)
    got2 = moe.combine(w, lay, eo.view(np.uint8).reshape(rx.shape), info, rng, topk, ntok, epoch=2)
    bonus = np.where(topk >= 0, topk + 1, 0).sum(axis=2).astype(np.uint32)
    want2 = (want + bonus[:, :, None]).astype(np.uint32)
    for p in range(P):
        want2[p, ntok[p]:] = 0
    assert np.array_equal(got2.view(np.uint32).reshape(P, T, Hb // 4), want2)


def test_combine_sum_wraps():
    P, E, T, K, Hb = 2, 2, 1, 2, 4
    topk = np.array([[[0, 1]], [[-1, -1]]], dtype=np.int32)
    ntok = np.array([1, 0], dtype=np.int32)
    x = np.zeros((P, T, Hb), dtype=np.uint8)
    x[0, 0] = np.array([0xFFFFFFF0], dtype=np.uint32).view(np.uint8)
    w, lay, (rx, info, rng, cnt) = run_dispatch(P, E, T, K, Hb, x, topk, ntok)
    got = moe.combine(w, lay, rx, info, rng, topk, ntok)
    assert got[0, 0].view(np.uint32)[0] == (2 * 0xFFFFFFF0) % (1 << 32)


def test_empty_batch_still_signals_every_pair():
    P, E, T, K, Hb = 3, 6, 4, 2, 8
    topk = np.full((P, T, K), -1, dtype=np.int32)
    ntok = np.zeros(P, dtype=np.int32)
    x = workgen.moe_tokens(9, P, T, Hb)
    w, lay, (rx, info, rng, cnt) = run_dispatch(P, E, T, K, Hb, x, topk, ntok)
    assert not cnt.any() and not rng.any() and not rx.any()
    got = moe.combine(w, lay, rx, info, rng, topk, ntok)
    assert not got.any()

"""GPU parity for the MoE-shaped dispatch / combine: the HIP kernels, called through the C ABI,
against the oracle on the same seeded routing tables and tokens, element by element (bit-exact:
this is byte and integer work).  Senders and receivers of one launch run on different dies, so a
receiver only packs fresh bytes if the count signal really follows the data."""
import numpy as np
import pytest
import torch

import oracle
import workgen
from oracle import moe as omoe

pytestmark = pytest.mark.gpu

sh = pytest.importorskip("paper_2511_15076_amd")
from gpu_util import as_np, shmem_world  # noqa: E402


def oracle_run(P, E, T, K, Hb, x, topk, ntok, rounds=1, mutate=None):
    lay = omoe.MoeLayout(P, E, T, K, Hb)
    w = oracle.World(P, lay.end, oracle.SHUFFLED, 5)
    for p in range(P):
        w.heap(p)[:] = 0
    outs = []
    for r in range(rounds):
        d = omoe.dispatch(w, lay, x, topk, ntok)
        eo = mutate(d[0], d[3]) if mutate else d[0]
        c = omoe.combine(w, lay, eo, d[1], d[2], topk, ntok, epoch=r + 1)
        outs.append((d, eo, c))
    return outs


def heap_bytes_for(P, E, T, K, Hb):
    epp = E // P
    up = lambda v: (v + 255) // 256 * 256
    return up(epp * P * T * (Hb + 16)) + up(T * K * Hb) + up(8 * (2 * E + 8)) + 4096


class DevMoe:
    def __init__(self, P, E, T, K, Hb):
        self.shape = (P, E, T, K, Hb)
        epp = E // P
        dev = "cuda:0"
        self.moe = sh.moe_create(E, T, K, Hb)
        self.recv_x = torch.zeros((P, epp, P * T, Hb), dtype=torch.uint8, device=dev)
        self.recv_info = torch.zeros((P, epp, P * T, 4), dtype=torch.int32, device=dev)
        self.recv_range = torch.zeros((P, epp, P, 2), dtype=torch.int32, device=dev)
        self.recv_count = torch.zeros((P, epp), dtype=torch.int32, device=dev)
        self.combined = torch.zeros((P, T, Hb), dtype=torch.uint8, device=dev)

    def dispatch(self, x, topk, ntok, wgs):
        self.x, self.topk, self.ntok = (torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0") for a in (x, topk, ntok))
        sh.moe_dispatch(self.moe, self.x, self.topk, self.ntok, self.recv_x, self.recv_info, self.recv_range,
                        self.recv_count, wgs)
        sh.stream_sync()
        return tuple(t.cpu().numpy() for t in (self.recv_x, self.recv_info, self.recv_range, self.recv_count))

    def combine(self, expert_out, wgs):
        eo = torch.from_numpy(np.ascontiguousarray(expert_out)).to("cuda:0")
        sh.moe_combine(self.moe, eo, self.recv_info, self.recv_range, self.topk, self.ntok, self.combined, wgs)
        sh.stream_sync()
        return self.combined.cpu().numpy()

    def close(self):
        sh.moe_destroy(self.moe)


def check_dispatch(got, want):
    (gx, gi, gr, gc), (wx, wi, wr, wc) = got, want
    assert np.array_equal(gc, wc)
    assert np.array_equal(gr, wr)
    P, epp = gc.shape
    for r in range(P):
        for le in range(epp):
            n = wc[r, le]
            assert np.array_equal(gi[r, le, :n], wi[r, le, :n]), (r, le)
            assert np.array_equal(gx[r, le, :n], wx[r, le, :n]), (r, le)
            assert not gx[r, le, n:].any()                     # rows beyond the count are never written


def bump(rx, cnt):
    """Stand-in expert: adds (global expert id + 1) to every 32-bit word of its rows."""
    P, epp = cnt.shape
    eo = rx.view(np.uint32).copy()
    for r in range(P):
        for le in range(epp):
            eo[r, le, :cnt[r, le]] += np.uint32(r * epp + le + 1)
    return eo.view(np.uint8)


CASES = [
    # P, E, T, K, Hb, ntok, dist, drop, wgs
    (2, 4, 3, 2, 16, None, "uniform", 0.0, 1),
    (4, 16, 16, 4, 272, [16, 0, 7, 16], "zipf", 0.2, 3),        # ragged: an empty PE, dropped entries, odd team size
    (8, 32, 128, 8, 1040, None, "uniform", 0.0, 8),             # full token count, several tiles per message
    (3, 9, 5, 9, 48, None, "uniform", 0.0, 2),                  # every token to every expert
    (8, 8, 128, 1, 2064, None, "zipf", 0.0, 16),                # one expert per PE, more workgroups than experts
    (16, 64, 33, 6, 528, None, "zipf", 0.1, 4),
    (1, 4, 9, 2, 16, None, "uniform", 0.0, 2),                 # a single PE talks to itself; smallest token
    (4, 64, 128, 64, 32, [128, 1, 77, 128], "uniform", 0.3, 5),  # widest top-k, every expert, ragged batches
    (2, 1024, 16, 8, 64, None, "zipf", 0.0, 7),                # the largest expert count
    # batches of 32 tokens and more per PE are shared out dynamically (fixed ranges + claimed blocks):
    (4, 8, 64, 2, 48, [64, 31, 32, 0], "uniform", 0.0, 1),      # both kinds of PE in one exchange, one workgroup per PE
    (2, 6, 40, 3, 80, None, "zipf", 1.0, 3),                   # every entry dropped: large batches with nothing to send
    (8, 16, 32, 1, 16, None, "uniform", 0.0, 64),              # more workgroups than messages: nothing fixed, every block claimed
    (3, 12, 100, 4, 14352, None, "zipf", 0.1, 11),             # long messages of an odd length, odd team size (a token limit
                                                               # that is no multiple of 8: the fixed split at every batch size)
    (3, 12, 104, 4, 14352, None, "zipf", 0.1, 11),             # the same shared out dynamically, packed pair by pair
    (5, 40, 48, 8, 1040, [48, 40, 0, 33, 48], "uniform", 0.2, 6),  # five PEs: the send order of every PE starts at its own experts
    (2, 128, 128, 64, 32, None, "uniform", 0.0, 1),            # 8192 routes per PE on ONE workgroup: more blocks of four than its
                                                               # list of ranges holds, so the blocks grow
    (2, 128, 128, 64, 32, [128, 97], "zipf", 0.1, 2),
]


def _random_case(seed):
    rng = np.random.default_rng(7000 + seed)
    P = int(rng.choice([1, 2, 3, 4, 5, 8]))
    epp = int(rng.choice([1, 2, 3, 5, 9]))
    E = P * epp
    T = int(rng.integers(1, 40))
    K = int(rng.integers(1, min(E, 8) + 1))
    Hb = 16 * int(rng.choice([1, 2, 3, 17, 64, 65, 129]))
    ntok = [int(rng.integers(0, T + 1)) for _ in range(P)]
    return (P, E, T, K, Hb, ntok, str(rng.choice(["uniform", "zipf"])), float(rng.choice([0.0, 0.0, 0.25])),
            int(rng.choice([1, 2, 3, 4, 7, 9])))


CASES += [_random_case(seed) for seed in range(8)]       # shapes nobody chose: sizes, raggedness and team sizes drawn at random


@pytest.mark.parametrize("P,E,T,K,Hb,ntok,dist,drop,wgs", CASES)
def test_dispatch_and_combine_match_oracle(P, E, T, K, Hb, ntok, dist, drop, wgs):
    topk, ntok = workgen.moe_routing(100 + P + E, P, E, T, K, ntok=ntok, dist=dist, drop=drop)
    x = workgen.moe_tokens(200 + T, P, T, Hb)
    rounds = 2
    want = oracle_run(P, E, T, K, Hb, x, topk, ntok, rounds=rounds, mutate=bump)
    with shmem_world(P, heap_bytes_for(P, E, T, K, Hb)):
        dm = DevMoe(P, E, T, K, Hb)
        for r in range(rounds):                                 # the second round reuses slots and signals
            got = dm.dispatch(x, topk, ntok, wgs)
            check_dispatch(got, want[r][0])
            eo = bump(got[0], got[3])
            assert np.array_equal(eo, want[r][1])
            comb = dm.combine(eo, wgs)
            assert np.array_equal(comb, want[r][2])
        dm.close()


def test_paper_message_size_single_token():
    # one token per PE, 7168 16-bit values = 14,336 bytes, 14,352-byte messages (Sec. V-C)
    P, E, T, K, Hb = 8, 288, 1, 8, 14336
    topk, ntok = workgen.moe_routing(7, P, E, T, K)
    x = workgen.moe_tokens(8, P, T, Hb)
    want = oracle_run(P, E, T, K, Hb, x, topk, ntok)
    with shmem_world(P, heap_bytes_for(P, E, T, K, Hb)):
        dm = DevMoe(P, E, T, K, Hb)
        got = dm.dispatch(x, topk, ntok, 32)
        check_dispatch(got, want[0][0])
        comb = dm.combine(got[0], 32)
        assert np.array_equal(comb, want[0][2])
        dm.close()


def test_bad_routing_is_reported_not_sent():
    P, E, T, K, Hb = 2, 4, 4, 2, 32
    topk, ntok = workgen.moe_routing(1, P, E, T, K)
    x = workgen.moe_tokens(2, P, T, Hb)
    with shmem_world(P, heap_bytes_for(P, E, T, K, Hb)):
        dm = DevMoe(P, E, T, K, Hb)
        bad = topk.copy()
        bad[1, 2, 0] = E + 3                                    # no such expert
        with pytest.raises(sh.ShmemError) as ei:
            dm.dispatch(x, bad, ntok, 2)
        assert ei.value.status == sh.ERR_DEVICE_FAULT
        dm.close()
    with shmem_world(P, heap_bytes_for(P, E, T, K, Hb)):       # the fault word is sticky: fresh world
        dm = DevMoe(P, E, T, K, Hb)
        dup = topk.copy()
        dup[0, 1, 1] = dup[0, 1, 0]                             # the same expert twice in one token
        with pytest.raises(sh.ShmemError):
            dm.dispatch(x, dup, ntok, 2)
        dm.close()


def test_argument_checks():
    with shmem_world(4, 1 << 20):
        for args in [(6, 4, 2, 64), (8, 129, 2, 64), (8, 4, 65, 64), (8, 4, 2, 24), (8, 4, 2, 0), (2048, 4, 2, 64)]:
            with pytest.raises(sh.ShmemError) as ei:
                sh.moe_create(*args)
            assert ei.value.status == sh.ERR_INVALID_ARG
        with pytest.raises(sh.ShmemError) as ei:
            sh.moe_create(8, 128, 8, 1 << 20)                   # does not fit the heap
        assert ei.value.status == sh.ERR_NOMEM
        m = sh.moe_create(8, 4, 2, 64)
        t = torch.zeros(4096, dtype=torch.uint8, device="cuda:0")
        with pytest.raises(sh.ShmemError):
            sh.moe_dispatch(m, t, t, t, t, t, t, t, 0)
        with pytest.raises(sh.ShmemError):
            sh.moe_dispatch(m, t, t, t, t, t, t, t, 100000)     # cannot be co-resident
        sh.moe_destroy(m)


def test_full_size_batch_as_benchmarked():
    # the largest cell bench.py times: 8 PEs, 288 experts, top-8, 128 tokens of 14,336 bytes per PE, with
    # the team sizes it uses (36 workgroups per PE for small batches, 32 -- one per CU -- or 64 for large ones);
    # the oracle affords the whole batch (8192 messages)
    P, E, T, K, Hb = 8, 288, 128, 8, 14336
    topk, ntok = workgen.moe_routing(npes=P, num_experts=E, max_tokens=T, topk=K, ntok=T)
    x = workgen.moe_tokens(npes=P, max_tokens=T, hidden_bytes=Hb)
    want = oracle_run(P, E, T, K, Hb, x, topk, ntok, rounds=1, mutate=bump)
    with shmem_world(P, heap_bytes_for(P, E, T, K, Hb)):
        dm = DevMoe(P, E, T, K, Hb)
        for wgs in (36, 32, 64):
            got = dm.dispatch(x, topk, ntok, wgs)
            check_dispatch(got, want[0][0])
            comb = dm.combine(bump(got[0], got[3]), wgs)
            assert np.array_equal(comb, want[0][2])
        # 100 workgroups per PE are more than the 256 compute units hold at once (two of these workgroups each, by
        # their registers): refused on the host, not left to run into its bounded waits
        with pytest.raises(sh.ShmemError) as ei:
            dm.dispatch(x, topk, ntok, 100)
        assert ei.value.status == sh.ERR_INVALID_ARG
        dm.close()

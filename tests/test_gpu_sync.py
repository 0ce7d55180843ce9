"""GPU parity for in-kernel ordering: put -> signal (the ring exchange of
Listing 2), the put-with-signal ping-pong, and barrier epochs.  These run as
persistent launches with teams on different dies, so a reader only sees fresh
data if quiet / signal / barrier really release and acquire at device scope."""
import numpy as np
import pytest
import torch

import oracle
import workgen

pytestmark = pytest.mark.gpu

sh = pytest.importorskip("paper_2511_15076_amd")
from gpu_util import as_np, heaps_of, shmem_world  # noqa: E402


def golden_ring_cases(golden_dir):
    return [tuple(map(int, l.split())) for l in open(f"{golden_dir}/ring_exchange.txt")
            if l.strip() and not l.startswith("#")]


def gin_offsets(hb_payload, nsig, nctr):
    """Where the library will place a Gin object's arrays when it is the first allocation after
    `hb_payload` bytes reserved by the test (first fit, 256-byte granules)."""
    sig_bytes = (nsig * 8 + 255) // 256 * 256
    return hb_payload, hb_payload + sig_bytes


@pytest.mark.parametrize("wgs,rounds", [(1, 1), (3, 1), (2, 25)])
def test_ring_exchange_matches_listing2(golden_dir, wgs, rounds):
    ring_cases(golden_ring_cases(golden_dir) + [(8, 65536 + 24), (16, 1000), (4, (1 << 20) + 4096 + 32)], wgs, rounds)


def ring_cases(cases, wgs, rounds):
    for n, ds in cases:
        span = n * ds
        send, recv = 0, (span + 255) // 256 * 256
        payload = 2 * recv                                    # bytes the test reserves with shmem_malloc
        nsig, nctr, sig_id, ctr_id = 4, 3, 2, 1
        sig_base, ctr_base = gin_offsets(payload, nsig, nctr)
        hb = (ctr_base + 256 + 255) // 256 * 256
        init = np.stack([workgen.random_words(300 + p + ds, hb // 8).view(np.uint8) for p in range(n)])
        init[:, sig_base:] = 0                                # what gin_create clears
        w = oracle.World(n, hb, oracle.SHUFFLED, 2)
        for p in range(n):
            w.heap(p)[:] = init[p]
        sig = sig_base + 8 * sig_id
        for _ in range(rounds):
            for r in range(n):                                # put with SignalInc{sig_id}
                peer = (r + 1) % n
                assert w.put(r, recv + r * ds, send + peer * ds, ds, peer) == 0
                assert w.signal_add(r, sig, 1, peer) == 0
            for p in range(n):                                # waitSignal(sig_id, 1); resetSignal(sig_id)
                assert int(w.heap(p)[sig:sig + 8].view(np.uint64)[0]) == 1
                w.heap(p)[sig:sig + 8] = 0
            w.barrier_all()
        with shmem_world(n, hb) as (heap, base):
            heap.copy_(torch.from_numpy(init.reshape(-1)))
            assert sh.malloc(payload) == base
            gin = sh.gin_create(nsig, nctr)
            assert sh.gin_signal_sym(gin, sig_id) == base + sig
            assert sh.gin_counter_sym(gin, ctr_id) == base + ctr_base + 8 * ctr_id
            assert sh.gin_signal_sym(gin, nsig) is None and sh.gin_counter_sym(gin, -1) is None
            sh.ring_exchange(base + recv, base + send, ds, gin, sig_id, ctr_id, rounds, wgs)
            sh.stream_sync()
            got = heaps_of(heap, n)
            sh.gin_destroy(gin)
        assert np.array_equal(got, w.heaps()), (n, ds)       # data delivered, signals and counters back to 0
        for p in range(n):                                    # the worked example, spelled out
            q = (p - 1 + n) % n
            assert np.array_equal(got[p][recv + q * ds: recv + (q + 1) * ds],
                                  init[q][send + p * ds: send + (p + 1) * ds])


@pytest.mark.parametrize("nbytes", [8, 128, 4096, 14352, 1 << 20])
def test_pingpong(nbytes):
    pingpong_case(4, nbytes, 200)


def pingpong_case(npes, nbytes, iters):
    pad = (nbytes + 255) // 256 * 256
    buf, payload = 0, 2 * pad
    sig_base, ctr_base = gin_offsets(payload, 1, 0)
    hb = (ctr_base + 256 + 255) // 256 * 256
    init = np.stack([workgen.random_words(900 + p, hb // 8).view(np.uint8) for p in range(npes)])
    init[:, sig_base:] = 0
    w = oracle.World(npes, hb, oracle.SHUFFLED, 3)
    for p in range(npes):
        w.heap(p)[:] = init[p]
    for _ in range(iters):
        w.put(0, buf, buf, nbytes, 1); w.signal_add(0, sig_base, 1, 1)
        w.put(1, buf + pad, buf, nbytes, 0); w.signal_add(1, sig_base, 1, 0)
    with shmem_world(npes, hb) as (heap, base):
        heap.copy_(torch.from_numpy(init.reshape(-1)))
        assert sh.malloc(payload) == base
        gin = sh.gin_create(1, 0)
        sh.pingpong(base + buf, nbytes, gin, 0, iters)
        sh.stream_sync()
        got = heaps_of(heap, npes)
        sh.gin_destroy(gin)
    assert np.array_equal(got, w.heaps())                     # both signals read `iters`
    assert np.array_equal(got[0][pad:pad + nbytes], init[0][:nbytes])   # the payload came back


# launches of up to 256 workgroups meet on one word, larger ones in two stages (team, then world)
@pytest.mark.parametrize("npes,wgs,rounds", [(16, 2, 10000), (64, 1, 2000), (5, 3, 3000), (16, 24, 500), (3, 100, 500)])
def test_barrier_epochs(npes, wgs, rounds):
    hb = 4096
    with shmem_world(npes, hb) as (heap, base):
        slots = sh.malloc(8 * npes)
        err = torch.zeros(1, dtype=torch.int64, device="cuda:0")
        sh.barrier_epochs(slots, rounds, wgs, err)
        sh.stream_sync()
        assert int(err.item()) == 0                            # nobody left a barrier early
        got = heaps_of(heap, npes)
        off = slots - base
    w = oracle.World(npes, hb, oracle.AT_QUIET, 0)
    assert w.malloc(8 * npes) == off
    for p in range(npes):                                     # the last round decides the final state
        for q in range(npes):
            w.put_value(p, off + 8 * p, rounds, 8, q)
    w.barrier_all()
    assert np.array_equal(got, w.heaps())


@pytest.mark.parametrize("use_quiet", [0, 1])
@pytest.mark.parametrize("nbytes", [8, 4096, 1 << 20])
def test_fence_and_quiet_order_data_before_the_flag(nbytes, use_quiet):
    # put data; fence (or quiet); put flag; quiet -- whoever sees the flag sees the data, 300 rounds between
    # two dies; a stale word would be counted
    npes, rounds = 3, 300
    pad = (nbytes + 255) // 256 * 256
    with shmem_world(npes, pad + 4096) as (heap, base):
        buf = sh.malloc(pad + 512)
        errors = torch.zeros(1, dtype=torch.int64, device="cuda:0")
        sh.fence_litmus(buf, nbytes, rounds, use_quiet, errors)
        sh.stream_sync()
        assert int(errors.item()) == 0
        got = heaps_of(heap, npes)
        off = buf - base
        assert (got[1, off:off + nbytes].view(np.uint64) == rounds).all()       # the last block arrived whole
        assert got[1, off + pad:off + pad + 8].view(np.uint64)[0] == rounds     # flag on PE 1
        assert got[0, off + pad + 256:off + pad + 264].view(np.uint64)[0] == rounds   # acknowledgement on PE 0
        assert not got[2].any()                                                  # a bystander PE is untouched
        for call in (lambda: sh.fence_litmus(buf, 12, 1), lambda: sh.fence_litmus(buf, 8, -1),
                     lambda: sh.fence_litmus(buf + pad, 1 << 20, 1)):
            with pytest.raises(sh.ShmemError):
                call()


def test_cooperative_launch_switch(monkeypatch):
    # MI_SHMEM_COOPERATIVE_LAUNCH=1 (read at init) launches the kernels with in-kernel waits cooperatively:
    # same results, the formal residency guarantee instead of the occupancy check alone
    monkeypatch.setenv("MI_SHMEM_COOPERATIVE_LAUNCH", "1")
    npes, wgs, rounds = 8, 3, 50
    with shmem_world(npes, 4096) as (heap, base):
        slots = sh.malloc(8 * npes)
        errors = torch.zeros(1, dtype=torch.int64, device="cuda:0")
        sh.barrier_epochs(slots, rounds, wgs, errors)
        sh.fence_litmus(sh.malloc(1024), 256, 20, 0, errors)
        sh.stream_sync()
        assert int(errors.item()) == 0
        off = slots - base
        assert (heaps_of(heap, npes)[:, off:off + 8 * npes].view(np.uint64) == rounds).all()


def test_sync_entry_point_errors():
    with shmem_world(4, 1 << 16) as (heap, base):
        gin = sh.gin_create(2, 1)
        for call, status in [
            (lambda: sh.ring_exchange(base, base + 128, 256, gin, 0, 0, 1, 1), sh.ERR_INVALID_ARG),     # overlap
            (lambda: sh.ring_exchange(base + 4096, base, 256, gin, 2, 0, 1, 1), sh.ERR_INVALID_ARG),    # signal id
            (lambda: sh.ring_exchange(base + 4096, base, 256, gin, 0, 1, 1, 1), sh.ERR_INVALID_ARG),    # counter id
            (lambda: sh.ring_exchange(base + 4096, base, 1 << 15, gin, 0, 0, 1, 1), sh.ERR_OUT_OF_RANGE),
            (lambda: sh.ring_exchange(base + 4096, base, 256, gin, 0, 0, 1, 100000), sh.ERR_INVALID_ARG),
            (lambda: sh.pingpong(base, 1 << 16, gin, 0, 1), sh.ERR_OUT_OF_RANGE),
            (lambda: sh.pingpong(base, 4096, gin, 5, 1), sh.ERR_INVALID_ARG),
            (lambda: sh.gin_create(0, 0), sh.ERR_INVALID_ARG),
            (lambda: sh.gin_create(1 << 19, 0), sh.ERR_NOMEM),
            (lambda: sh.barrier_epochs(base + 4, 1, 1), sh.ERR_ALIGN),
            (lambda: sh.barrier_epochs(base, 1, 0), sh.ERR_INVALID_ARG),
        ]:
            with pytest.raises(sh.ShmemError) as e:
                call()
            assert e.value.status == status
        sh.gin_destroy(gin)
        sh.stream_sync()


def test_a_timed_out_wait_leaves_the_library_usable():
    """After a bounded wait has given up, arrival counts and generations are half-advanced.  The state is planted
    from the host (no kernel is made to hang): a time-out code in the fault word, stale arrivals on the world
    barrier, on a PE's team words, on a team object's words and on a Gin signal.  shmem_stream_sync reports the
    fault once and starts all of it afresh; barriers and signal waits then work as after shmem_init."""
    npes, hb = 8, 1 << 16
    dev = torch.device("cuda:0")
    heap = torch.zeros(npes * hb, dtype=torch.uint8, device=dev)
    scratch = torch.zeros(sh.scratch_bytes(npes), dtype=torch.uint8, device=dev)
    sh.init(npes, hb, heap, scratch, torch.cuda.current_stream().cuda_stream)
    try:
        base = heap.data_ptr()
        slots = sh.malloc(8 * npes)
        gin = sh.gin_create(2, 1)
        team = sh.team_create(0, 2, 4)
        sig_off = sh.gin_signal_sym(gin, 0) - base
        team_off = int(sh.team_device_state(team).words_off)
        words = scratch.view(torch.int64)
        hv = heap.view(npes, hb)
        words[0] = 2                      # DEV_ERR_BARRIER_TIMEOUT
        words[1] = 5                      # the workgroup that gave up
        words[16] = 3                     # three stale arrivals on the world barrier
        words[32] = 41                    # ... and a generation somewhere in the middle
        words[64 + 64 * 2] = 1            # PE 2's team barrier: one stale arrival
        words[64 + 64 * 2 + 32] = 1       # and its stage of the world barrier
        hv[0, team_off:team_off + 8].view(torch.int64)[0] = 2          # the team object: two of four arrived
        hv[1, sig_off:sig_off + 8].view(torch.int64)[0] = 9            # a signal that was never reset
        torch.cuda.synchronize()
        with pytest.raises(sh.ShmemError) as ei:
            sh.stream_sync()
        assert ei.value.status == sh.ERR_DEVICE_FAULT and ei.value.first_bad_index == 5
        torch.cuda.synchronize()
        assert int(words.abs().sum().item()) == 0
        assert int(hv[0, team_off:team_off + 256].sum().item()) == 0 and int(hv[1, sig_off:sig_off + 8].sum().item()) == 0
        sh.stream_sync()                  # reported once
        errors = torch.zeros(1, dtype=torch.int64, device=dev)
        sh.barrier_epochs(slots, 200, 4, errors)
        sh.team_epochs([team], [150], slots, 2, errors)
        recv, send = sh.malloc(8 * 256), sh.malloc(8 * 256)
        sh.ring_exchange(recv, send, 256, gin, 0, 0, 20, 2)
        sh.stream_sync()
        assert int(errors.item()) == 0
        sh.team_destroy(team)
        sh.gin_destroy(gin)
    finally:
        sh.finalize()

"""Barriers over teams of PEs (start, stride, size): several disjoint teams run side by side in one
persistent launch, each for its own number of rounds, which a world barrier could not do; the final heap
is the oracle's, and no member ever leaves a barrier before the others' puts of that round are visible."""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu

sh = pytest.importorskip("paper_2511_15076_amd")
from gpu_util import heaps_of, shmem_world  # noqa: E402


def members(t):
    start, stride, size = t
    return [start + i * stride for i in range(size)]


CASES = [
    # npes, wgs, [(start, stride, size), rounds] ...
    (12, 2, [((0, 2, 4), 700), ((1, 4, 3), 300), ((3, 1, 1), 5)]),          # 7, 8, 10, 11 belong to no team
    (8, 1, [((0, 1, 8), 400)]),                                             # the team of everybody
    (16, 3, [((0, 2, 8), 150), ((1, 2, 8), 1000)]),                         # evens and odds at different paces
    (9, 4, [((6, 1, 3), 50), ((0, 3, 2), 0), ((1, 1, 2), 333), ((4, 1, 1), 9)]),   # a team with no rounds at all
    (64, 2, [((0, 1, 32), 120), ((32, 2, 16), 77), ((33, 2, 16), 300)]),
]


@pytest.mark.parametrize("npes,wgs,plan", CASES)
def test_team_epochs_match_oracle(npes, wgs, plan):
    hb = 1 << 14
    w = oracle.World(npes, hb, oracle.AT_QUIET, 0)
    blocks = [w.malloc(256) for _ in plan]                    # where the library puts each team's words
    slots = w.malloc(8 * npes)
    for (t, rounds) in plan:                                  # the last round decides the final state
        if rounds:
            for i, p in enumerate(members(t)):
                for q in members(t):
                    assert w.put_value(p, slots + 8 * i, rounds, 8, q) == 0
            assert w.team_sync(*t) == 0
    assert all(w.pending(p) == 0 for p in range(npes))
    want = w.heaps().copy()
    with shmem_world(npes, hb) as (heap, base):
        teams = [sh.team_create(*t) for (t, _) in plan]
        for tm, (t, _), blk in zip(teams, plan, blocks):
            st = sh.team_device_state(tm)
            assert (st.start, st.stride, st.size, st.words_off) == (*t, blk)
        d_slots = sh.malloc(8 * npes)
        assert d_slots - base == slots
        err = torch.zeros(1, dtype=torch.int64, device="cuda:0")
        for rep in range(2):                                   # the second call starts from the first one's generations
            sh.team_epochs(teams, [r for (_, r) in plan], d_slots, wgs, err)
            sh.stream_sync()
        assert int(err.item()) == 0                            # nobody left a barrier early
        got = heaps_of(heap, npes).copy()
        for tm in teams:
            sh.team_sync(tm, wgs)                              # the barrier as a launch of its own
        sh.stream_sync()
        for tm in teams:
            sh.team_destroy(tm)
        assert sh.malloc(256 * len(plan)) == base              # the teams' blocks came back (and coalesced)
    for blk in blocks:                                         # the teams' own words (arrivals, generation) are the library's
        got[:, blk:blk + 256] = 0
    assert np.array_equal(got, want)
    for (t, rounds) in plan:
        for p in members(t):
            assert (got[p, slots:slots + 8 * t[2]].view(np.uint64) == rounds).all()


def test_team_argument_checks():
    with shmem_world(6, 1 << 14) as (heap, base):
        for args, status in [((0, 1, 7), sh.ERR_INVALID_PE), ((2, 2, 3), sh.ERR_INVALID_PE), ((-1, 1, 2), sh.ERR_INVALID_ARG),
                             ((0, 0, 2), sh.ERR_INVALID_ARG), ((0, 1, 0), sh.ERR_INVALID_ARG)]:
            with pytest.raises(sh.ShmemError) as e:
                sh.team_create(*args)
            assert e.value.status == status
        a, b = sh.team_create(0, 2, 3), sh.team_create(2, 1, 2)         # 0, 2, 4 and 2, 3: PE 2 is in both
        slots = sh.malloc(64)
        for call, status in [(lambda: sh.team_epochs([a, b], [3, 3], slots, 1), sh.ERR_INVALID_ARG),
                             (lambda: sh.team_epochs([a], [-1], slots, 1), sh.ERR_INVALID_ARG),
                             (lambda: sh.team_epochs([a] * 9, [1] * 9, slots, 1), sh.ERR_INVALID_ARG),
                             (lambda: sh.team_epochs([a], [1], slots + 4, 1), sh.ERR_ALIGN),
                             (lambda: sh.team_epochs([a], [1], slots, 100000), sh.ERR_INVALID_ARG),
                             (lambda: sh.team_sync(a, 0), sh.ERR_INVALID_ARG)]:
            with pytest.raises(sh.ShmemError) as e:
                call()
            assert e.value.status == status
        sh.team_epochs([], [], slots, 1)                                # nothing to do
        sh.team_epochs([a], [0], slots, 1)
        sh.team_epochs([a], [4], slots, 2)                              # and the teams still work
        sh.team_epochs([b], [6], slots, 1)
        sh.stream_sync()
        got = heaps_of(heap, 6)
        off = slots - base
        assert (got[[0, 4], off:off + 24].view(np.uint64) == 4).all()
        assert (got[3, off:off + 16].view(np.uint64) == 6).all() and (got[2, off:off + 16].view(np.uint64) == 6).all()
        sh.team_destroy(a); sh.team_destroy(b)

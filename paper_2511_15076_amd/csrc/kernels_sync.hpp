// Kernels that exercise in-kernel ordering through the GIN-shaped device API
// (include/mi_shmem_gin.hpp): put with a signal action, waitSignal, counters, the barrier
// session, and barrier epochs.  They are the device forms of the paper's ring
// exchange (Listing 2) and put-with-signal ping-pong (Sec. V-A).
#pragma once
#include "../../include/mi_shmem.h"
#include "../../include/mi_shmem_gin.hpp"
#include "../../include/mi_shmemx.hpp"

namespace shmemx {

// Ring exchange (Listing 2) through the GIN-shaped device API: PE r puts its
// send slot `peer` into slot r of the receive buffer of peer = (r+1) mod n with
// a SignalInc on signal `sig` (and a CounterInc on counter `ctr`), waits until
// its own signal shows the predecessor's arrival and resets it.  Rounds are
// separated by the barrier session, so a reset cannot swallow the next round's
// increment.
__global__ __launch_bounds__(256) void k_ring_exchange(Ctx c, GinState gs, uint64_t recv_off, uint64_t send_off,
                                                       uint64_t ds, uint32_t sig, uint32_t ctr, uint32_t rounds,
                                                       uint32_t wgs_per_pe)
{
    const uint32_t pe = blockIdx.x / wgs_per_pe, wg = blockIdx.x % wgs_per_pe;
    const Gin gin{c, gs, pe, wgs_per_pe};
    const uint32_t peer = (pe + 1) % (uint32_t)c.npes;
    for (uint32_t r = 1; r <= rounds; ++r) {
        GinActions act;
        act.signal_id = (int32_t)sig;               // SignalInc{sig}
        act.counter_id = (int32_t)ctr;              // CounterInc{ctr}
        gin.put(peer, recv_off + (uint64_t)pe * ds, send_off + (uint64_t)peer * ds, ds, act);
        gin.wait_signal(sig, 1);                    // the predecessor's data has arrived and is visible
        gin.wait_counter(ctr, r);                   // our own send slot is reusable
        team_barrier(c, pe, wgs_per_pe);            // every workgroup of the team has seen the signal ...
        if (wg == 0 && threadIdx.x == 0) gin.reset_signal(sig);   // ... so it can be reset
        gin.barrier_sync();
    }
    if (wg == 0 && threadIdx.x == 0) gin.reset_counter(ctr);
}

// Ping-pong between PE 0 and PE 1, one workgroup each (they run on different
// dies): PE 0 puts nbytes into PE 1's buffer with a SignalInc; PE 1 waits, puts
// the bytes it received back into PE 0's second buffer with a SignalInc;
// `iters` round trips.  The signal counts up; the host resets it.
__global__ __launch_bounds__(256) void k_pingpong(Ctx c, GinState gs, uint64_t buf_off, uint64_t nbytes, uint32_t sig,
                                                  uint32_t iters)
{
    const uint32_t pe = blockIdx.x;  // 0 or 1
    const Gin gin{c, gs, pe, 1};
    const uint64_t back_off = buf_off + ((nbytes + 255) / 256) * 256;
    GinActions act;
    act.signal_id = (int32_t)sig;
    for (uint32_t i = 1; i <= iters; ++i) {
        if (pe == 0) {
            gin.put(1, buf_off, buf_off, nbytes, act);
            gin.wait_signal(sig, i);
        } else {
            gin.wait_signal(sig, i);
            gin.put(0, back_off, buf_off, nbytes, act);
        }
    }
}

// Message-passing litmus for fence / quiet (Sec. III-A "Ordering semantics"; the put -> flag form of the
// paper's put -> signal rule): PE 0 and PE 1, one workgroup each, on different dies.  Round r: PE 0 fills
// its copy of the data block with r and puts it to PE 1 (whole workgroup), every wave orders its part with
// fence() -- or quiet() -- the workgroup meets, and ONE lane puts the 8-byte flag = r and makes it leave
// with quiet().  PE 1 polls its flag, acquires, and checks that every data word is r; then it puts the
// acknowledgement r back and PE 0, which waits for it, starts the next round.  A reader that sees the
// flag but not the data is counted in *errors.  Layout at buf_off: data (nbytes), then the flag and the
// acknowledgement word on lines of their own.
__global__ __launch_bounds__(256) void k_fence_litmus(Ctx c, uint64_t buf_off, uint64_t nbytes, uint32_t rounds,
                                                      int use_quiet, uint64_t *errors)
{
    const uint32_t pe = blockIdx.x;  // 0 or 1
    const uint64_t words = nbytes / 8;
    const uint64_t flag_off = buf_off + (nbytes + 255) / 256 * 256, ack_off = flag_off + 256;
    uint64_t *mine = (uint64_t *)ptr(c, buf_off, pe);
    uint64_t *my_flag = (uint64_t *)ptr(c, flag_off, pe), *my_ack = (uint64_t *)ptr(c, ack_off, pe);
    uint64_t bad = 0;
    for (uint32_t r = 1; r <= rounds; ++r) {
        if (pe == 0) {
            for (uint64_t i = threadIdx.x; i < words; i += blockDim.x) mine[i] = r;
            __syncthreads();                                  // the source is complete before anybody copies from it
            put(c, buf_off, (const uint8_t *)mine, nbytes, 1, threadIdx.x, blockDim.x);
            if (use_quiet) quiet(); else fence();             // every wave: its puts come before what follows
            __syncthreads();
            if (threadIdx.x == 0) {
                *my_flag = r;                                 // local source word of the flag put
                put(c, flag_off, (const uint8_t *)my_flag, 8, 1, 0, 1);
                quiet();                                      // delivery of the flag itself
                uint32_t spins = 0;
                while (atomic_fetch(my_ack) < r) {
                    if (timed_out(c, spins)) break;
                    __builtin_amdgcn_s_sleep(1);
                    if (++spins > SPIN_LIMIT) { report(c, DEV_ERR_BARRIER_TIMEOUT, r); break; }
                }
            }
            __syncthreads();
        } else {
            if (threadIdx.x == 0) {
                uint32_t spins = 0;
                while (atomic_fetch(my_flag) < r) {
                    if (timed_out(c, spins)) break;
                    __builtin_amdgcn_s_sleep(1);
                    if (++spins > SPIN_LIMIT) { report(c, DEV_ERR_BARRIER_TIMEOUT, r); break; }
                }
                acquire();
            }
            wg_acquire();
            for (uint64_t i = threadIdx.x; i < words; i += blockDim.x)
                if (*(volatile uint64_t *)(mine + i) != r) ++bad;
            __syncthreads();                                  // everybody has read before the sender may overwrite
            if (threadIdx.x == 0) {
                *my_ack = r;
                put(c, ack_off, (const uint8_t *)my_ack, 8, 0, 0, 1);
                quiet();
            }
        }
    }
    if (bad && errors) atomic_fetch_add(errors, bad);
}

// Clears the signal and counter arrays of a new Gin object on every PE.
__global__ void k_gin_zero(Ctx c, GinState gs)
{
    for (uint32_t pe = blockIdx.x; pe < (uint32_t)c.npes; pe += gridDim.x) {
        for (uint32_t i = threadIdx.x; i < gs.nsignals; i += blockDim.x) *(uint64_t *)ptr(c, gs.signals_off + 8ull * i, pe) = 0;
        for (uint32_t i = threadIdx.x; i < gs.ncounters; i += blockDim.x) *(uint64_t *)ptr(c, gs.counters_off + 8ull * i, pe) = 0;
    }
}

// Barrier epochs: in round e every PE puts the value e into word `pe` of the
// slot array on EVERY PE, all teams meet in barrier_all, then every PE reads
// its own copy of the array: each word must be at least e.  Violations are
// counted in *errors.
__global__ __launch_bounds__(256) void k_barrier_epochs(Ctx c, uint64_t slots_off, uint32_t rounds,
                                                        uint32_t wgs_per_pe, uint64_t *errors)
{
    const uint32_t pe = blockIdx.x / wgs_per_pe, wg = blockIdx.x % wgs_per_pe;
    const uint32_t npes = (uint32_t)c.npes;
    const uint32_t rank = wg * blockDim.x + threadIdx.x, size = wgs_per_pe * blockDim.x;
    uint64_t bad = 0;
    for (uint32_t e = 1; e <= rounds; ++e) {
        for (uint32_t q = rank; q < npes; q += size)                       // putValue to every PE
            *(uint64_t *)ptr(c, slots_off + 8ull * pe, q) = e;
        barrier_all(c, pe, wgs_per_pe);
        for (uint32_t q = rank; q < npes; q += size)
            if (*(volatile uint64_t *)ptr(c, slots_off + 8ull * q, pe) < e) ++bad;
    }
    if (bad && errors) atomic_fetch_add(errors, bad);
}

// One barrier of a team of PEs as a launch of its own (the members' workgroups meet; the others leave at once).
__global__ __launch_bounds__(256) void k_team_sync(Ctx c, PeTeam t, uint32_t wgs_per_pe)
{
    const uint32_t pe = blockIdx.x / wgs_per_pe;
    if (t.has(pe)) pe_team_sync(c, t, pe, wgs_per_pe);
}

// Team epochs: several disjoint teams of PEs run side by side in one launch, each for its own number of
// rounds.  In round e every member puts the value e into word (its index in the team) of the slot array on
// EVERY member, the team meets in its barrier, and every member checks that each word of its own copy is at
// least e.  A world barrier could not do this: the teams do not take the same number of rounds.
constexpr uint32_t TEAM_EPOCHS_MAX = 8;
struct TeamEpochsArgs {
    PeTeam team[TEAM_EPOCHS_MAX];
    uint32_t rounds[TEAM_EPOCHS_MAX];
    uint32_t nteams, wgs_per_pe;
    uint64_t slots_off;
    uint64_t *errors;
};

__global__ __launch_bounds__(256) void k_team_epochs(Ctx c, TeamEpochsArgs a)
{
    const uint32_t pe = blockIdx.x / a.wgs_per_pe, wg = blockIdx.x % a.wgs_per_pe;
    uint32_t ti = a.nteams;
    for (uint32_t k = 0; k < a.nteams; ++k)
        if (a.team[k].has(pe)) ti = k;
    if (ti == a.nteams) return;                                           // this PE is in none of the teams
    const PeTeam t = a.team[ti];
    const uint32_t me = t.index_of(pe);
    const uint32_t rank = wg * blockDim.x + threadIdx.x, size = a.wgs_per_pe * blockDim.x;
    uint64_t bad = 0;
    for (uint32_t e = 1; e <= a.rounds[ti]; ++e) {
        for (uint32_t q = rank; q < t.size; q += size)                      // putValue to every member
            *(uint64_t *)ptr(c, a.slots_off + 8ull * me, t.member(q)) = e;
        pe_team_sync(c, t, pe, a.wgs_per_pe);
        for (uint32_t q = rank; q < t.size; q += size)
            if (*(volatile uint64_t *)ptr(c, a.slots_off + 8ull * q, pe) < e) ++bad;
    }
    if (bad && a.errors) atomic_fetch_add(a.errors, bad);
}

}  // namespace shmemx

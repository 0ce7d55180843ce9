// Kernels that exercise in-kernel ordering through the GIN-shaped device API
// (gin.hpp): put with a signal action, waitSignal, counters, the barrier
// session, and barrier epochs.  They are the device forms of the paper's ring
// exchange (Listing 2) and put-with-signal ping-pong (Sec. V-A).
#pragma once
#include "../../include/mi_shmem.h"
#include "gin.hpp"
#include "shmemx.hpp"

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

}  // namespace shmemx

// Kernels that exercise in-kernel ordering: put followed by a signal (a remote
// atomic add that makes the earlier puts visible), waiting on a signal, and
// barrier epochs.  They are the device forms of the paper's ring exchange
// (Listing 2) and put-with-signal ping-pong (Sec. V-A).
#pragma once
#include "../../include/mi_shmem.h"
#include "shmemx.hpp"

namespace shmemx {

// signal: remote atomic add on a 64-bit signal word of PE pe.  Called by one
// lane after the wave (or, behind a team barrier, the team) has issued its
// puts: the release makes every earlier put of the caller visible before the
// add lands (Sec. III-A "Ordering semantics").
__device__ __forceinline__ void signal_add(const Ctx &c, uint64_t sig_off, uint64_t value, uint32_t pe)
{
    __hip_atomic_fetch_add((uint64_t *)ptr(c, sig_off, pe), value, __ATOMIC_RELEASE, SHMEMX_AGENT);
}

// waitSignal: spin (relaxed polls) until the local signal word reaches `expected`;
// the caller then acquires so that the data the signal announces is read fresh.  Bounded; returns false
// on time-out (the fault word is set and the caller carries on).
__device__ __forceinline__ bool wait_signal(const Ctx &c, uint64_t sig_off, uint64_t expected, uint32_t pe_self)
{
    const uint64_t *w = (const uint64_t *)ptr(c, sig_off, pe_self);
    bool ok = true;
    uint32_t spins = 0;
    while (__hip_atomic_load(w, __ATOMIC_RELAXED, SHMEMX_AGENT) < expected) {   // the caller acquires afterwards
        if (timed_out(c)) { ok = false; break; }
        __builtin_amdgcn_s_sleep(1);
        if (++spins > SPIN_LIMIT) { report(c, DEV_ERR_BARRIER_TIMEOUT, pe_self); ok = false; break; }
    }
    return ok;
}

// Ring exchange: PE r puts its send slot `peer` into slot r of the receive
// buffer of peer = (r+1) mod n, increments the peer's signal, waits for its own
// signal to show this round's arrival, and after the last round resets it.
__global__ __launch_bounds__(256) void k_ring_exchange(Ctx c, uint64_t recv_off, uint64_t send_off, uint64_t ds,
                                                       uint64_t sig_off, uint32_t rounds, uint32_t wgs_per_pe)
{
    const uint32_t pe = blockIdx.x / wgs_per_pe, wg = blockIdx.x % wgs_per_pe;
    const uint32_t npes = (uint32_t)c.npes, peer = (pe + 1) % npes;
    const size_t rank = (size_t)wg * blockDim.x + threadIdx.x, size = (size_t)wgs_per_pe * blockDim.x;
    for (uint32_t r = 1; r <= rounds; ++r) {
        put(c, recv_off + (uint64_t)pe * ds, ptr(c, send_off + (uint64_t)peer * ds, pe), ds, peer, rank, size);
        team_barrier(c, pe, wgs_per_pe);                 // every wave's puts are complete and visible
        if (wg == 0 && threadIdx.x == 0) signal_add(c, sig_off, 1, peer);
        if (threadIdx.x == 0) wait_signal(c, sig_off, r, pe);
        __syncthreads();
        acquire();
    }
    barrier_all(c, pe, wgs_per_pe);                      // nobody still waits on a signal ...
    if (wg == 0 && threadIdx.x == 0)                     // ... so it can be reset for the next use
        __hip_atomic_store((uint64_t *)ptr(c, sig_off, pe), 0ull, __ATOMIC_RELAXED, SHMEMX_AGENT);
}

// Ping-pong between PE 0 and PE 1, one workgroup each (they run on different
// dies): PE 0 puts nbytes into PE 1's buffer and signals; PE 1 waits, puts the
// bytes it received back into PE 0's second buffer and signals; `iters` times.
// Signals count up; the host resets them.
__global__ __launch_bounds__(256) void k_pingpong(Ctx c, uint64_t buf_off, uint64_t nbytes, uint64_t sig_off,
                                                  uint32_t iters)
{
    const uint32_t pe = blockIdx.x;  // 0 or 1
    const uint64_t back_off = buf_off + ((nbytes + 255) / 256) * 256;
    for (uint32_t i = 1; i <= iters; ++i) {
        if (pe == 0) {
            put(c, buf_off, ptr(c, buf_off, 0), nbytes, 1, threadIdx.x, blockDim.x);
            quiet();
            __syncthreads();
            if (threadIdx.x == 0) { signal_add(c, sig_off, 1, 1); wait_signal(c, sig_off, i, 0); }
            __syncthreads();
            acquire();
        } else {
            if (threadIdx.x == 0) wait_signal(c, sig_off, i, 1);
            __syncthreads();
            acquire();
            put(c, back_off, ptr(c, buf_off, 1), nbytes, 0, threadIdx.x, blockDim.x);
            quiet();
            __syncthreads();
            if (threadIdx.x == 0) signal_add(c, sig_off, 1, 0);
        }
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

// Device-side API in the shape of the paper's simplified GIN interface
// (Listing 1): put with optional completion actions, putValue, signal,
// flush, ID-addressed signals (symmetric, remote completion) and counters
// (local completion), and a barrier over the world team.  Here a "window" is
// the symmetric heap itself, addressed by byte offset; a signal / counter ID is
// an index into two small symmetric uint64 arrays owned by the Gin object.
#pragma once
#include "mi_shmemx.hpp"

namespace shmemx {

struct GinState {            // host-created, passed to kernels by value
    uint64_t signals_off;    // symmetric uint64[nsignals]
    uint64_t counters_off;   // uint64[ncounters] in every PE's segment (each PE uses its own)
    uint32_t nsignals, ncounters;
};

// Completion actions attached to a put (Listing 1, "Optional: attach completion actions").
struct GinActions {
    int32_t signal_id = -1;     // >= 0: add signal_value to that signal on the peer once the data is visible
    uint64_t signal_value = 1;  // 1 = SignalInc, anything else = SignalAdd
    int32_t counter_id = -1;    // >= 0: increment that local counter once the source is reusable
};

struct Gin {
    Ctx c;
    GinState g;
    uint32_t pe;             // the calling PE
    uint32_t wgs_per_pe;     // workgroups in its team

    __device__ __forceinline__ uint64_t *signal_word(uint32_t id, uint32_t on_pe) const
    {
        return (uint64_t *)ptr(c, g.signals_off + 8ull * id, on_pe);
    }
    __device__ __forceinline__ uint64_t *counter_word(uint32_t id) const
    {
        return (uint64_t *)ptr(c, g.counters_off + 8ull * id, pe);
    }

    // put by the whole team: bytes from the caller's window offset src_off to the peer's window
    // offset dst_off.  With actions, the team first makes the data visible (team barrier), then one
    // lane performs them; the signal therefore lands only after the put is visible at the peer
    // (Sec. III-A "Ordering semantics").  Every thread of every workgroup of the team must call it.
    __device__ __forceinline__ void put(uint32_t peer, uint64_t dst_off, uint64_t src_off, uint64_t bytes,
                                        const GinActions &a = GinActions()) const
    {
        const size_t wg = blockIdx.x % wgs_per_pe;
        shmemx::put(c, dst_off, ptr(c, src_off, pe), bytes, peer, wg * blockDim.x + threadIdx.x,
                    (size_t)wgs_per_pe * blockDim.x);
        if (a.signal_id < 0 && a.counter_id < 0) return;
        team_barrier(c, pe, wgs_per_pe);
        if (wg == 0 && threadIdx.x == 0) {
            if (a.signal_id >= 0 && (uint32_t)a.signal_id < g.nsignals)
                __hip_atomic_fetch_add(signal_word((uint32_t)a.signal_id, peer), a.signal_value, __ATOMIC_RELEASE,
                                       SHMEMX_AGENT);
            if (a.counter_id >= 0 && (uint32_t)a.counter_id < g.ncounters)
                __hip_atomic_fetch_add(counter_word((uint32_t)a.counter_id), 1ull, __ATOMIC_RELAXED, SHMEMX_AGENT);
        }
    }

    // putValue: a small inline value, no source buffer (one lane).
    __device__ __forceinline__ void put_value(uint32_t peer, uint64_t dst_off, uint64_t value) const
    {
        __hip_atomic_store((uint64_t *)ptr(c, dst_off, peer), value, __ATOMIC_RELAXED, SHMEMX_AGENT);
    }

    // signal: remote atomic add (one lane); earlier puts of the calling wave are visible before it lands.
    __device__ __forceinline__ void signal(uint32_t peer, uint32_t id, uint64_t value = 1) const
    {
        if (id < g.nsignals) __hip_atomic_fetch_add(signal_word(id, peer), value, __ATOMIC_RELEASE, SHMEMX_AGENT);
    }

    // flush: local completion only -- the sources of the calling wave's puts are reusable.  It makes
    // no promise about remote visibility (the paper's flush, unlike quiet).
    __device__ __forceinline__ void flush() const { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup"); }

    __device__ __forceinline__ uint64_t read_signal(uint32_t id) const
    {
        return __hip_atomic_load(signal_word(id, pe), __ATOMIC_RELAXED, SHMEMX_AGENT);
    }
    __device__ __forceinline__ uint64_t read_counter(uint32_t id) const
    {
        return __hip_atomic_load(counter_word(id), __ATOMIC_RELAXED, SHMEMX_AGENT);
    }

    // waitSignal / waitCounter by a workgroup: thread 0 polls (bounded), everybody acquires.
    __device__ __forceinline__ void wait_word(const uint64_t *w, uint64_t expected) const
    {
        if (threadIdx.x == 0) {
            uint32_t spins = 0;
            while (__hip_atomic_load(w, __ATOMIC_RELAXED, SHMEMX_AGENT) < expected) {
                if (timed_out(c, spins)) break;
                __builtin_amdgcn_s_sleep(1);
                if (++spins > SPIN_LIMIT) { report(c, DEV_ERR_BARRIER_TIMEOUT, pe); break; }
            }
            acquire();
        }
        wg_acquire();
    }
    __device__ __forceinline__ void wait_signal(uint32_t id, uint64_t expected) const
    {
        wait_word(signal_word(id, pe), expected);
    }
    __device__ __forceinline__ void wait_counter(uint32_t id, uint64_t expected) const
    {
        wait_word(counter_word(id), expected);
    }
    __device__ __forceinline__ void reset_signal(uint32_t id) const
    {
        __hip_atomic_store(signal_word(id, pe), 0ull, __ATOMIC_RELAXED, SHMEMX_AGENT);
    }
    __device__ __forceinline__ void reset_counter(uint32_t id) const
    {
        __hip_atomic_store(counter_word(id), 0ull, __ATOMIC_RELAXED, SHMEMX_AGENT);
    }

    // barrier session over the world team, or over a team of PEs that the caller is a member of
    __device__ __forceinline__ void barrier_sync() const { barrier_all(c, pe, wgs_per_pe); }
    __device__ __forceinline__ void barrier_sync(const PeTeam &team) const { pe_team_sync(c, team, pe, wgs_per_pe); }
};

}  // namespace shmemx

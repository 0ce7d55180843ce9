// Streaming copy for bandwidth-bound put / get: wave-specialised workgroups, one per compute unit, that
// move their team's list of 4 KiB tasks through a ring in LDS.
//
//   * Four READER waves fetch with the global-load-to-LDS instruction of gfx950 (16 bytes per lane, 1 KiB
//     per wave instruction): the data never occupies vector registers, so one wave keeps a dozen loads in
//     flight and a compute unit has 60 KiB of reads outstanding with four waves.
//   * Two WRITER waves drain the ring (ds_read_b128, then 16-byte non-temporal stores).  Writes reach
//     their best rate with few waves per compute unit and a compact chip-wide window, which is what
//     256 workgroups x one 4 KiB task per step give (1 MiB per step).
//   * One s_barrier per task orders the two sides; the readers run RING - 1 tasks ahead.
//   * The workgroup is PACED by the constant-rate clock: wave 0 lets the barrier of a task go no earlier
//     than one period after the previous one (lateness of up to one period is made up for, beyond that the
//     schedule starts afresh), and the loads of the next task follow the barrier.  Left to itself -- every
//     load issued as soon as a ring slot is free -- the copy drives the memory system into a congested
//     regime that delivers about 5.5 TB/s however deep or shallow the ring; asked for slightly less than it
//     can sustain (about 6.8 TB/s of read + write traffic on this chip) it delivers what it is asked for.
//
// The task list of a team: task t = (op, chunk), op = t / chunks_per_op, chunk = t % chunks_per_op,
// slot = op % nslots; workgroup `rank` of `team` takes the tasks (rank + j * team + rot) mod ntasks.
// `rot` differs from PE to PE (an odd multiple of the task size) so that teams that walk identically
// laid out windows in step do not keep meeting in the same memory channels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/mi_shmem.h"
#include "../../include/mi_shmemx.hpp"

namespace shmemx {

constexpr uint32_t ST_CHUNK = 4096;       // one task: four 1 KiB rows, one per reader wave
constexpr uint32_t ST_READERS = 4;
constexpr uint32_t ST_WRITERS = 2;
constexpr uint32_t ST_RING = 16;          // tasks in the LDS ring (64 KiB)
constexpr uint32_t ST_THREADS = (ST_READERS + ST_WRITERS) * 64;
constexpr uint32_t ST_ROT = 13;           // PE p starts (13 * p) mod ntasks tasks into its list

typedef __attribute__((address_space(3))) void *lds_ptr_t;
typedef const __attribute__((address_space(1))) void *glb_ptr_t;

// s_waitcnt vmcnt(n) alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, the other counters left at their maxima)
#define ST_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (7 << 4) | (15 << 8) | ((((n) >> 4) & 3) << 14))
// a wave-uniform value, kept in a scalar register
#define ST_UNIFORM(x) ((uint32_t)__builtin_amdgcn_readfirstlane((int)(x)))

struct StreamPlan {
    const uint8_t *src;
    uint8_t *dst;
    uint64_t spitch, dpitch;    // slot pitches in bytes
    uint32_t cpo;               // chunks per op
    uint32_t nslots;
    uint32_t ntasks;            // cpo * ops, below 2^32
    uint32_t team, rank;        // workgroups of the team, this workgroup's number
    uint32_t rot;               // below ntasks
    uint32_t period;            // pacing: 1/256 ticks of the constant-rate clock per task; 0 = unpaced
};

// (chunk, slot) of the workgroup's current task, advanced without divisions
struct StreamWalker {
    uint32_t ch, slot, step_ch, step_slot, tau;
    __device__ __forceinline__ void seek(uint32_t cpo, uint32_t nslots, uint32_t t)
    {
        tau = t;
        const uint32_t op = t / cpo;
        ch = ST_UNIFORM(t - op * cpo);
        slot = ST_UNIFORM(op % nslots);
    }
    __device__ __forceinline__ void init(const StreamPlan &p)
    {
        step_ch = ST_UNIFORM(p.team % p.cpo);
        step_slot = ST_UNIFORM((p.team / p.cpo) % p.nslots);
        uint32_t t = p.rank + p.rot;
        if (t >= p.ntasks || t < p.rank) t -= p.ntasks;
        seek(p.cpo, p.nslots, ST_UNIFORM(t));
    }
    __device__ __forceinline__ void next(const StreamPlan &p)
    {
        const uint32_t nt = tau + p.team;
        if (__builtin_expect(nt >= p.ntasks || nt < tau, 0)) { seek(p.cpo, p.nslots, nt - p.ntasks); return; }   // the rotation wraps once
        tau = nt;
        ch += step_ch; slot += step_slot;
        if (ch >= p.cpo) { ch -= p.cpo; slot += 1; }
        if (slot >= p.nslots) slot -= p.nslots;
    }
};

// Every wave of the workgroup calls this with the same plan; `ring` is ST_RING * ST_CHUNK bytes of LDS.
__device__ __forceinline__ void stream_copy(const StreamPlan &p, uint8_t *ring)
{
    constexpr uint32_t S = ST_RING;
    static_assert((S & (S - 1)) == 0 && S >= 4 && S - 2 <= 63, "ring: a power of two, and vmcnt counts to 63");
    const uint32_t lane16 = (threadIdx.x & 63) * 16;
    const uint32_t wave = ST_UNIFORM(threadIdx.x >> 6);
    if (p.rank >= p.ntasks) return;                                   // the whole workgroup leaves together
    const uint32_t T = (p.ntasks - 1 - p.rank) / p.team + 1;         // tasks of this workgroup
    StreamWalker w;
    w.init(p);
    if (wave < ST_READERS) {
        const uint32_t row_off = wave * 1024;
        auto issue = [&](uint32_t t) {
            const uint8_t *g = p.src + (uint64_t)w.slot * p.spitch + (uint64_t)w.ch * ST_CHUNK + row_off + lane16;
            uint8_t *l = ring + (t & (S - 1)) * ST_CHUNK + row_off;   // lane i lands at l + 16 i
            __builtin_amdgcn_global_load_lds((glb_ptr_t)g, (lds_ptr_t)l, 16, 0, 2 /* nt */);
            w.next(p);
        };
        const uint32_t pro = T < S - 1 ? T : S - 1;
        for (uint32_t t = 0; t < pro; ++t) issue(t);
        // Where in its period this workgroup issues: spread over the workgroups, so that after a stall that
        // stops the whole chip for a microsecond or two (they happen) the workgroups do not all come back in step.
        const uint64_t phase = ((uint64_t)p.period * ((blockIdx.x * 167u) & 255u)) >> 8;
        uint64_t next_issue = 0;
        for (uint32_t t = 0; t < T; ++t) {
            // task t has landed once at most the loads of the S - 2 tasks after it are outstanding
            // (loads return in order); near the end, where fewer follow, wait for everything
            if (t + (S - 1) < T) ST_WAIT_VM(S - 2); else ST_WAIT_VM(0);
            if (p.period && wave == 0 && t + (S - 1) < T) {
                // Wave 0 holds the workgroup's barrier back until the next loads are due (average-rate pacing:
                // lateness of up to one period is made up for by the following tasks; beyond that the
                // schedule starts afresh rather than answering a stall with a burst).
                uint64_t now = __builtin_amdgcn_s_memrealtime() << 8;
                if (t == 0) next_issue = now + phase;
                while (now < next_issue) { __builtin_amdgcn_s_sleep(1); now = __builtin_amdgcn_s_memrealtime() << 8; }
                if (now > next_issue + p.period) next_issue = now + phase;
                next_issue += p.period;
            }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();        // writers: task t is theirs; slot (t - 1) mod S has been read out
            asm volatile("" ::: "memory");
            if (t + (S - 1) < T) issue(t + (S - 1));
        }
    } else {
        constexpr uint32_t PER = ST_READERS / ST_WRITERS;              // rows per writer
        const uint32_t wr = wave - ST_READERS;
        for (uint32_t t = 0; t < T; ++t) {
            uint8_t *d = p.dst + (uint64_t)w.slot * p.dpitch + (uint64_t)w.ch * ST_CHUNK + lane16;
            w.next(p);
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            const uint8_t *l = ring + (t & (S - 1)) * ST_CHUNK + lane16;
            u32x4 v[PER];
#pragma unroll
            for (uint32_t j = 0; j < PER; ++j) v[j] = *(const u32x4 *)(l + (wr + j * ST_WRITERS) * 1024);
#pragma unroll
            for (uint32_t j = 0; j < PER; ++j) __builtin_nontemporal_store(v[j], (u32x4 *)(d + (wr + j * ST_WRITERS) * 1024));
            // the stores have taken their data out of the registers the ds_reads filled, so every read of
            // this slot is complete before the wave reaches the next barrier
        }
    }
}

// Bandwidth-sweep cell through the streaming copy: contiguous messages that are whole multiples of
// ST_CHUNK with 16-byte aligned placement.  PE team p = workgroups [p * team, (p + 1) * team).
struct StreamSweepArgs {
    int kind;                   // SHMEM_OP_PUT / SHMEM_OP_GET
    uint64_t remote_off, local_off, count, remote_slot, local_slot;
    uint32_t nslots, ops_per_pe, team, period;
};

__global__ __launch_bounds__(ST_THREADS) void k_copy_sweep_stream(Ctx c, StreamSweepArgs a)
{
    __shared__ __attribute__((aligned(16))) uint8_t ring[ST_RING * ST_CHUNK];
    const uint32_t pe = blockIdx.x / a.team, peer = (pe + 1) % (uint32_t)c.npes;
    uint8_t *const lbase = ptr(c, a.local_off, pe);
    uint8_t *const rbase = ptr(c, a.remote_off, peer);
    const bool is_put = a.kind == SHMEM_OP_PUT;
    StreamPlan p;
    p.src = is_put ? lbase : rbase;
    p.dst = is_put ? rbase : lbase;
    p.spitch = is_put ? a.local_slot : a.remote_slot;
    p.dpitch = is_put ? a.remote_slot : a.local_slot;
    p.cpo = (uint32_t)(a.count / ST_CHUNK);
    p.nslots = a.nslots;
    p.ntasks = p.cpo * a.ops_per_pe;
    p.team = a.team; p.rank = blockIdx.x % a.team;
    p.rot = (uint32_t)(((uint64_t)ST_ROT * pe) % p.ntasks);
    p.period = a.period;
    stream_copy(p, ring);
}

// One contiguous copy of `chunks` whole chunks: the grid is one team.
__global__ __launch_bounds__(ST_THREADS) void k_copy_stream_lds(uint8_t *__restrict__ dst, const uint8_t *__restrict__ src,
                                                                uint32_t chunks, uint32_t period)
{
    __shared__ __attribute__((aligned(16))) uint8_t ring[ST_RING * ST_CHUNK];
    StreamPlan p;
    p.src = src; p.dst = dst; p.spitch = p.dpitch = 0;
    p.cpo = chunks; p.nslots = 1; p.ntasks = chunks;
    p.team = gridDim.x; p.rank = blockIdx.x; p.rot = 0; p.period = period;
    stream_copy(p, ring);
}

}  // namespace shmemx

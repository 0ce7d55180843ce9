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

// ---------------------------------------------------------------------------------------------------
// The same copy with the team's task list handed out DYNAMICALLY: a workgroup claims blocks of ST_BLOCK
// consecutive tasks from a per-team counter (one returning atomic add per block, issued two blocks ahead of
// its use by a seventh wave that also does the pacing).  A workgroup that the memory system serves more
// slowly then simply takes fewer blocks: the launch ends when the work is done instead of when the slowest
// workgroup has walked its fixed share, and the tasks in flight stay a compact window however far the
// workgroups' rates drift apart.
//
// The first ST_STATIC blocks of a workgroup are fixed (rank, rank + team, ...), so loading starts without
// waiting for a claim; the counter hands out blocks from ST_STATIC * team on.  Block numbers travel to the
// reader and writer waves through a small queue in LDS; the end (the first claim beyond the last block) is
// published at least ST_RING steps before the last task, so every wave runs the same number of barriers.
constexpr uint32_t ST_BLOCK = 4;
constexpr uint32_t ST_STATIC = 4;        // ST_STATIC * ST_BLOCK >= ST_RING: the prologue needs no claim
constexpr uint32_t ST_QUEUE = 16;        // block numbers kept in LDS (a power of two)
constexpr uint32_t ST_DYN_THREADS = ST_THREADS + 64;
// s_waitcnt lgkmcnt(0) alone
#define ST_WAIT_LGKM0() __builtin_amdgcn_s_waitcnt(15 | (7 << 4) | (0 << 8) | (3 << 14))

// tasks of one block, in order: (chunk, slot) advanced by one
struct BlockWalker {
    uint32_t ch, slot, tau, left, j;
    __device__ __forceinline__ void start(const StreamPlan &p, uint32_t block)
    {
        uint32_t t = block * ST_BLOCK + p.rot;                // below 2^32: ntasks < 2^31
        if (t >= p.ntasks) t -= p.ntasks;
        tau = ST_UNIFORM(t);
        const uint32_t op = tau / p.cpo;
        ch = ST_UNIFORM(tau - op * p.cpo);
        slot = ST_UNIFORM(op % p.nslots);
        left = ST_BLOCK;
    }
    __device__ __forceinline__ void next(const StreamPlan &p)
    {
        --left; ++tau; ++ch;
        if (ch == p.cpo) { ch = 0; ++slot; if (slot == p.nslots) slot = 0; }
        if (tau == p.ntasks) { tau = 0; ch = 0; slot = 0; }
    }
};

// For messages that are not whole multiples of 4 KiB the dynamic copy works on ROWS of 1 KiB (one wave
// instruction; the last row of a message may be short), so that messages of any length pack into full tasks: the
// team's list is the rows of all its operations in order, a task is four consecutive rows (one per reader wave,
// two per writer wave), a block ST_BLOCK tasks.  Whole multiples of 4 KiB keep the task walk above: the row walk
// costs them a few per cent (it sits closer to the edge of the congested regime at the same pace).
struct StreamRows {
    const uint8_t *src;
    uint8_t *dst;
    uint64_t spitch, dpitch;    // slot pitches in bytes
    uint32_t rpo;               // rows per operation, the last of which may be short:
    uint32_t tail;              // its bytes (a multiple of 16, at most 1024)
    uint32_t step_r, step_s;    // four rows on: 4 % rpo rows and 4 / rpo operations (kept so that a step needs no loop)
    uint32_t nslots;
    uint32_t nrows;             // rpo * operations, below 2^31; the last block may be short
    uint32_t team, rank;
    uint32_t rot;               // the team starts rot rows into its list (below nrows)
    uint32_t period;            // pacing per task, as in StreamPlan
};

// Every fourth row of a block, from row `w` of its first task on: (row in its operation, slot) advanced by four
// rows.  Position u of the list (block * 16 + ...) is row (u + rot) mod nrows; a position from nrows on, in the
// last block, stands for position 0 once more: that row is then moved a second time, the same bytes to the same
// place, and every wave keeps exactly one load or two stores per step.
struct RowWalker {
    uint32_t r, slot, rho, u, left, j;
    __device__ __forceinline__ void seek(const StreamRows &p, uint32_t at)
    {
        rho = ST_UNIFORM(at);
        const uint32_t op = rho / p.rpo;
        r = ST_UNIFORM(rho - op * p.rpo);
        slot = ST_UNIFORM(op % p.nslots);
    }
    __device__ __forceinline__ void start(const StreamRows &p, uint32_t block, uint32_t w)
    {
        u = ST_UNIFORM(block * (4 * ST_BLOCK) + w);
        uint32_t at = (u < p.nrows ? u : 0) + p.rot;          // below 2^32: nrows < 2^31
        if (at >= p.nrows) at -= p.nrows;
        seek(p, at);
        left = ST_BLOCK;
    }
    __device__ __forceinline__ void next(const StreamRows &p)
    {
        --left; u += 4; rho += 4;
        if (__builtin_expect(u >= p.nrows, 0)) { seek(p, p.rot); return; }               // beyond the list
        if (__builtin_expect(rho >= p.nrows, 0)) { seek(p, rho - p.nrows); return; }     // the rotation wraps once
        r += p.step_r; slot += p.step_s;
        if (r >= p.rpo) { r -= p.rpo; ++slot; }
        if (slot >= p.nslots) { slot -= p.nslots; if (slot >= p.nslots) slot %= p.nslots; }   // (fewer than five slots)
    }
};

// Messages of 256 or 512 bytes (any power of two from 16 up would do): a row is 1024 / count consecutive operations (their slots are consecutive,
// the host sees to it that a row never wraps round the slots), walked as one operation of one row whose slot
// pitch is that of the whole group; inside the row every lane adds the place of its own message.
struct StreamPacked : StreamRows {
    uint32_t lane_s, lane_d;    // this lane's 16 bytes inside the group, on the source and on the destination side
};

template <class Plan> struct StreamWalk;
template <> struct StreamWalk<StreamPlan> { typedef BlockWalker type; };
template <> struct StreamWalk<StreamRows> { typedef RowWalker type; };
template <> struct StreamWalk<StreamPacked> { typedef RowWalker type; };

typedef __attribute__((address_space(3))) uint32_t lds_u32_t;
typedef __attribute__((address_space(1))) uint64_t glb_u64_t;

// Two LDS words read by a wave that has global-load-to-LDS instructions in flight.  Written as one asm
// statement with its own wait: an LDS read the compiler can see makes it wait for every outstanding
// load-to-LDS first (they might alias), which would serialise the ring.
__device__ __forceinline__ void lds_read_pair(uint32_t addr_a, uint32_t addr_b, uint32_t &a, uint32_t &b)
{
    asm volatile("ds_read_b32 %0, %2\n\tds_read_b32 %1, %3\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(a), "=&v"(b) : "v"(addr_a), "v"(addr_b) : "memory");
}

// `claim`: the team's counter, `done`: one word for the whole launch; both zero at launch and zero again at
// its end (`claim0`, `nteams`, `claim_stride`: all the launch's counters, for the workgroup that finishes last).
// `ring`: ST_RING * ST_CHUNK bytes of LDS, `q`: ST_QUEUE block numbers and one word for the end, in LDS.
// Plan = StreamPlan: whole 4 KiB tasks (ntasks a multiple of ST_BLOCK); Plan = StreamRows: rows, as above.
template <class Plan>
__device__ __forceinline__ void stream_copy_dyn(const Plan &p, uint64_t *claim, uint64_t *done, uint64_t *claim0,
                                                uint32_t nteams, uint32_t claim_stride, uint8_t *ring, uint32_t *q_generic)
{
    constexpr uint32_t S = ST_RING, B = ST_BLOCK, Q = ST_QUEUE;
    constexpr bool PACKED = __is_same(Plan, StreamPacked);
    constexpr bool ROWS = __is_same(Plan, StreamRows) || PACKED;
    static_assert(ST_STATIC * B >= S && (Q & (Q - 1)) == 0 && Q >= ST_STATIC + S / B + 4, "queue and static prefix cover the read-ahead");
    volatile lds_u32_t *const q = (volatile lds_u32_t *)q_generic;
    const uint32_t lane16 = (threadIdx.x & 63) * 16;
    const uint32_t wave = ST_UNIFORM(threadIdx.x >> 6);
    uint32_t nblocks;                                                 // host: nblocks >= 2 * ST_STATIC * team
    if constexpr (ROWS) nblocks = (p.nrows + 4 * B - 1) / (4 * B); else nblocks = p.ntasks / B;   // (tasks: whole blocks)
    if (threadIdx.x < ST_STATIC) q[threadIdx.x] = p.rank + threadIdx.x * p.team;
    if (threadIdx.x == 0) q[Q] = 0xffffffffu;
    __syncthreads();
    uint32_t T = 0xffffffffu;                                         // tasks of this workgroup, once its end is known
    if (wave < ST_READERS) {
        const uint32_t row_off = wave * 1024;
        const uint32_t qaddr = (uint32_t)(uintptr_t)q;
        typename StreamWalk<Plan>::type w;
        w.left = 0; w.j = 0;
        uint32_t issued = 0;
        auto issue = [&]() {
            if (w.left == 0) {
                uint32_t blk, te;
                lds_read_pair(qaddr + 4 * (w.j & (Q - 1)), qaddr + 4 * Q, blk, te);
                T = ST_UNIFORM(te);
                if (issued >= T) return;                              // the workgroup's last block has been issued
                if constexpr (ROWS) w.start(p, ST_UNIFORM(blk), wave); else w.start(p, ST_UNIFORM(blk));
                ++w.j;
            }
            const uint8_t *g;
            if constexpr (PACKED) {
                g = p.src + (uint64_t)w.slot * p.spitch + p.lane_s;
            } else if constexpr (ROWS) {
                // (the lanes beyond a short last row fetch its last vector once more: nothing is predicated, and the
                // writers, which do the same, put the same bytes in the same place)
                const uint32_t at = min(lane16, (w.r + 1 == p.rpo ? p.tail : 1024u) - 16);
                g = p.src + (uint64_t)w.slot * p.spitch + (uint64_t)w.r * 1024 + at;
            } else {
                g = p.src + (uint64_t)w.slot * p.spitch + (uint64_t)w.ch * ST_CHUNK + row_off + lane16;
            }
            uint8_t *l = ring + (issued & (S - 1)) * ST_CHUNK + row_off;
            __builtin_amdgcn_global_load_lds((glb_ptr_t)g, (lds_ptr_t)l, 16, 0, 2 /* nt */);
            w.next(p);
            ++issued;
        };
        for (uint32_t t = 0; t < S - 1; ++t) issue();
        for (uint32_t t = 0; t < T; ++t) {
            // task t has landed once at most the S - 2 loads issued after it are outstanding
            if (issued - t - 1 >= S - 2) ST_WAIT_VM(S - 2); else ST_WAIT_VM(0);
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            issue();
        }
    } else if (wave < ST_READERS + ST_WRITERS) {
        constexpr uint32_t PER = ST_READERS / ST_WRITERS;
        const uint32_t wr = wave - ST_READERS;
        if constexpr (ROWS) {
            static_assert(PER == 2, "a writer wave walks two rows of every task");
            RowWalker wa, wb;                                         // rows wr and wr + ST_WRITERS of every task
            wa.left = 0; wa.j = 0;
            for (uint32_t t = 0; t < T; ++t) {
                if (wa.left == 0) {
                    T = ST_UNIFORM(q[Q]);                             // published at least ST_RING steps before it matters
                    const uint32_t blk = ST_UNIFORM(q[wa.j & (Q - 1)]);
                    wa.start(p, blk, wr);
                    wb.start(p, blk, wr + ST_WRITERS);
                    ++wa.j;
                }
                uint8_t *da, *db;
                if constexpr (PACKED) {
                    da = p.dst + (uint64_t)wa.slot * p.dpitch + p.lane_d;
                    db = p.dst + (uint64_t)wb.slot * p.dpitch + p.lane_d;
                } else {
                    da = p.dst + (uint64_t)wa.slot * p.dpitch + (uint64_t)wa.r * 1024 + min(lane16, (wa.r + 1 == p.rpo ? p.tail : 1024u) - 16);
                    db = p.dst + (uint64_t)wb.slot * p.dpitch + (uint64_t)wb.r * 1024 + min(lane16, (wb.r + 1 == p.rpo ? p.tail : 1024u) - 16);
                }
                wa.next(p); wb.next(p);
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                const uint8_t *l = ring + (t & (S - 1)) * ST_CHUNK + lane16;
                const u32x4 va = *(const u32x4 *)(l + wr * 1024), vb = *(const u32x4 *)(l + (wr + ST_WRITERS) * 1024);
                __builtin_nontemporal_store(va, (u32x4 *)da);
                __builtin_nontemporal_store(vb, (u32x4 *)db);
            }
        } else {
            BlockWalker w;
            w.left = 0; w.j = 0;
            for (uint32_t t = 0; t < T; ++t) {
                if (w.left == 0) {
                    T = ST_UNIFORM(q[Q]);                             // published at least ST_RING steps before it matters
                    w.start(p, ST_UNIFORM(q[w.j & (Q - 1)]));
                    ++w.j;
                }
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
            }
        }
    } else {
        // The scheduler wave: claims blocks two ahead of their use, publishes them, and paces the barrier.
        const bool lead = (threadIdx.x & 63) == 0;
        // The counter's address goes through a vector register the compiler cannot see through: an atomic on
        // an address it knows to be uniform is rewritten into a wave-wide reduction whose result is read at
        // once, which would make every claim a full round trip in this wave.
        uint64_t craw = (uint64_t)claim;
        asm volatile("" : "+v"(craw));
        glb_u64_t *const cp = (glb_u64_t *)craw;
        const uint64_t phase = ((uint64_t)p.period * ((blockIdx.x * 167u) & 255u)) >> 8;
        uint64_t next_issue = 0, cA = 0, cB = 0;
        if (lead) {
            cA = __hip_atomic_fetch_add(cp, 1ull, __ATOMIC_RELAXED, SHMEMX_AGENT);
            cB = __hip_atomic_fetch_add(cp, 1ull, __ATOMIC_RELAXED, SHMEMX_AGENT);
        }
        uint32_t j = ST_STATIC, t = 0;
        bool ended = false;
        // B paced barriers
        auto steps = [&]() {
            for (uint32_t i = 0; i < B && t < T; ++i, ++t) {
                if (p.period && t + (S - 1) < T) {
                    uint64_t now = __builtin_amdgcn_s_memrealtime() << 8;
                    if (t == 0) next_issue = now + phase;
                    while (now < next_issue) { __builtin_amdgcn_s_sleep(1); now = __builtin_amdgcn_s_memrealtime() << 8; }
                    if (now > next_issue + p.period) next_issue = now + phase;
                    next_issue += p.period;
                }
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
            }
        };
        // One block: publish block j = ST_STATIC + t / B of this workgroup from the claim `c` made two turns ago
        // (the readers look for it after barrier t + 1), make the next claim into `c`, run the block's barriers.
        // Called for cA and cB in turn, so that each claim has its own register and nothing waits for the newest.
        auto turn = [&](uint64_t &c) {
            if (!ended) {
                const uint64_t b = (uint64_t)ST_UNIFORM((uint32_t)c) + (uint64_t)ST_STATIC * p.team;   // counts stay below 2^31
                if (b >= nblocks) {
                    ended = true;
                    T = j * B;
                    if (lead) q[Q] = T;
                } else {
                    if (lead) q[j & (Q - 1)] = (uint32_t)b;
                    ++j;
                }
                ST_WAIT_LGKM0();
                if (!ended && lead) c = __hip_atomic_fetch_add(cp, 1ull, __ATOMIC_RELAXED, SHMEMX_AGENT);
            }
            steps();
        };
        while (t < T) { turn(cA); turn(cB); }
        if (lead) {
            // every claim of this workgroup has returned (both values are read) before it counts itself done;
            // the last workgroup of the launch puts the counters back to zero for the next launch
            const uint64_t seen = cA + cB;
            asm volatile("" :: "v"(seen) : "memory");
            const uint64_t d = __hip_atomic_fetch_add(done, 1ull, __ATOMIC_RELAXED, SHMEMX_AGENT);
            if (d + 1 == gridDim.x) {
                for (uint32_t i = 0; i < nteams; ++i) __hip_atomic_store(claim0 + (uint64_t)i * claim_stride, 0ull, __ATOMIC_RELAXED, SHMEMX_AGENT);
                __hip_atomic_store(done, 0ull, __ATOMIC_RELAXED, SHMEMX_AGENT);
            }
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

// The same cell with dynamic task claiming (ntasks a multiple of ST_BLOCK, at least 2 * ST_STATIC blocks per
// workgroup, fewer than 2^31 tasks).  The claim counter of PE p is word 8 of the PE's first scratch line (no
// barrier runs in this kernel), the launch's done count a general-purpose scratch word.
__global__ __launch_bounds__(ST_DYN_THREADS) void k_copy_sweep_stream_dyn(Ctx c, StreamSweepArgs a)
{
    __shared__ __attribute__((aligned(16))) uint8_t ring[ST_RING * ST_CHUNK];
    __shared__ uint32_t q[ST_QUEUE + 1];
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
    uint64_t *const claim0 = &c.scratch[W_PE_BASE + 8];
    stream_copy_dyn(p, claim0 + (uint64_t)pe * W_PE_WORDS, &c.scratch[W_WORK + 8], claim0, (uint32_t)c.npes, W_PE_WORDS, ring, q);
}

// Dynamic claiming for messages of 1 KiB rows of which the last may be short (any 16-byte multiple from 1 KiB
// up): at least 2 * ST_STATIC blocks of rows per workgroup, fewer than 2^31 rows.  Same counters.
__global__ __launch_bounds__(ST_DYN_THREADS) void k_copy_sweep_stream_rows(Ctx c, StreamSweepArgs a)
{
    __shared__ __attribute__((aligned(16))) uint8_t ring[ST_RING * ST_CHUNK];
    __shared__ uint32_t q[ST_QUEUE + 1];
    const uint32_t pe = blockIdx.x / a.team, peer = (pe + 1) % (uint32_t)c.npes;
    uint8_t *const lbase = ptr(c, a.local_off, pe);
    uint8_t *const rbase = ptr(c, a.remote_off, peer);
    const bool is_put = a.kind == SHMEM_OP_PUT;
    StreamRows p;
    p.src = is_put ? lbase : rbase;
    p.dst = is_put ? rbase : lbase;
    p.spitch = is_put ? a.local_slot : a.remote_slot;
    p.dpitch = is_put ? a.remote_slot : a.local_slot;
    p.rpo = (uint32_t)((a.count + 1023) / 1024);
    p.tail = (uint32_t)(a.count - (uint64_t)(p.rpo - 1) * 1024);
    p.step_r = 4 % p.rpo; p.step_s = 4 / p.rpo;
    p.nslots = a.nslots;
    p.nrows = p.rpo * a.ops_per_pe;
    p.team = a.team; p.rank = blockIdx.x % a.team;
    p.rot = (uint32_t)(((uint64_t)ST_ROT * 4 * pe) % p.nrows);
    p.period = a.period;
    uint64_t *const claim0 = &c.scratch[W_PE_BASE + 8];
    stream_copy_dyn(p, claim0 + (uint64_t)pe * W_PE_WORDS, &c.scratch[W_WORK + 8], claim0, (uint32_t)c.npes, W_PE_WORDS, ring, q);
}

// Dynamic claiming for messages of 256 or 512 bytes (a power of two below 1024), 1024 / count of them per row (ops_per_pe and nslots are
// multiples of that, the group's pitch is below 2^32; at least 2 * ST_STATIC blocks of rows per workgroup).
__global__ __launch_bounds__(ST_DYN_THREADS) void k_copy_sweep_stream_packed(Ctx c, StreamSweepArgs a)
{
    __shared__ __attribute__((aligned(16))) uint8_t ring[ST_RING * ST_CHUNK];
    __shared__ uint32_t q[ST_QUEUE + 1];
    const uint32_t pe = blockIdx.x / a.team, peer = (pe + 1) % (uint32_t)c.npes;
    uint8_t *const lbase = ptr(c, a.local_off, pe);
    uint8_t *const rbase = ptr(c, a.remote_off, peer);
    const bool is_put = a.kind == SHMEM_OP_PUT;
    const uint32_t count = (uint32_t)a.count, per_row = 1024 / count, lane16 = (threadIdx.x & 63) * 16;
    const uint64_t spitch = is_put ? a.local_slot : a.remote_slot, dpitch = is_put ? a.remote_slot : a.local_slot;
    StreamPacked p;
    p.src = is_put ? lbase : rbase;
    p.dst = is_put ? rbase : lbase;
    p.spitch = spitch * per_row;
    p.dpitch = dpitch * per_row;
    p.lane_s = (uint32_t)((lane16 / count) * spitch) + lane16 % count;
    p.lane_d = (uint32_t)((lane16 / count) * dpitch) + lane16 % count;
    p.rpo = 1; p.tail = 1024;
    p.step_r = 0; p.step_s = 4;
    p.nslots = a.nslots / per_row;
    p.nrows = a.ops_per_pe / per_row;
    p.team = a.team; p.rank = blockIdx.x % a.team;
    p.rot = (uint32_t)(((uint64_t)ST_ROT * 4 * pe) % p.nrows);
    p.period = a.period;
    uint64_t *const claim0 = &c.scratch[W_PE_BASE + 8];
    stream_copy_dyn(p, claim0 + (uint64_t)pe * W_PE_WORDS, &c.scratch[W_WORK + 8], claim0, (uint32_t)c.npes, W_PE_WORDS, ring, q);
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

// Device-side one-sided primitives for gfx950 (wave64).  Every call takes a
// cooperation scope -- the (rank, size) of the calling lane among the lanes
// that perform the operation together (one lane, a wavefront, a workgroup or a
// whole PE team) -- mirroring the `coop` argument of the paper's device API
// (Listing 1; Sec. I "cooperation models").
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace shmemx {

// Kernel-argument view of the symmetric heap.
struct Ctx {
    uint8_t *heap;      // PE 0's segment
    uint64_t seg;       // bytes per PE segment
    uint64_t *scratch;  // library scratch words (layout below)
    int npes;
};

// Scratch layout in 64-bit words.  Words that are spun on or hammered by
// atomics sit alone on a 128-byte line.
enum : uint32_t {
    W_ERR_FLAG = 0,     // 0 = no device fault, else a DEV_ERR_* code
    W_ERR_INDEX = 1,    // index of the first rejected op
    W_BAR_COUNT = 16,   // world barrier: arrivals
    W_BAR_GEN = 32,     // world barrier: generation
    W_WORK = 48,        // 16 general-purpose counters (BFS edge sum, ...)
    W_PE_BASE = 64,     // per PE: 64 words; +0 / +16 team barrier arrivals / generation,
    W_PE_WORDS = 64     //               +32 / +48 the team's stage of the world barrier
};
enum : uint64_t { DEV_ERR_BAD_OP = 1, DEV_ERR_BARRIER_TIMEOUT = 2, DEV_ERR_BAD_TARGET = 3 };

#define SHMEMX_AGENT __HIP_MEMORY_SCOPE_AGENT

__device__ __forceinline__ uint8_t *ptr(const Ctx &c, uint64_t off, uint32_t pe)
{
    return c.heap + (uint64_t)pe * c.seg + off;
}

__device__ __forceinline__ void report(const Ctx &c, uint64_t code, uint64_t index)
{
    unsigned long long expect = 0;
    if (__hip_atomic_compare_exchange_strong((unsigned long long *)&c.scratch[W_ERR_FLAG], &expect,
                                             (unsigned long long)code, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                             SHMEMX_AGENT))
        __hip_atomic_store(&c.scratch[W_ERR_INDEX], index, __ATOMIC_RELAXED, SHMEMX_AGENT);
}

constexpr uint32_t SPIN_LIMIT = 1u << 20;  // polls before a device-side wait gives up

// true once some wait of this launch has timed out
__device__ __forceinline__ bool timed_out(const Ctx &c)
{
    return __hip_atomic_load(&c.scratch[W_ERR_FLAG], __ATOMIC_RELAXED, SHMEMX_AGENT) == DEV_ERR_BARRIER_TIMEOUT;
}
// The same, looked at only on every 64th poll of a wait loop: the fault word costs a round trip to
// memory like the polled word itself, and the two cannot overlap.
__device__ __forceinline__ bool timed_out(const Ctx &c, uint32_t spins)
{
    return (spins & 63) == 63 && timed_out(c);
}

// ---------------------------------------------------------------------------
// Atomic memory operations (Table II "memory atomics"): agent scope, so that
// workgroups on different XCDs (separate L2s) resolve them at one point.
__device__ __forceinline__ uint64_t atomic_fetch_add(uint64_t *p, uint64_t v)
{
    return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, SHMEMX_AGENT);
}
// A returning fetch-add whose result is looked at LATER (a claim of work made ahead of its use).  The address
// goes through a vector register the compiler cannot see through: an atomic on an address it knows to be
// wave-uniform is rewritten into a wave-wide reduction whose result is read at once, which turns the claim
// into a synchronous round trip.
__device__ __forceinline__ uint64_t atomic_fetch_add_deferred(uint64_t *p, uint64_t v)
{
    typedef __attribute__((address_space(1))) uint64_t global_u64;
    uint64_t raw = (uint64_t)p;
    asm volatile("" : "+v"(raw));
    return __hip_atomic_fetch_add((global_u64 *)raw, v, __ATOMIC_RELAXED, SHMEMX_AGENT);
}
__device__ __forceinline__ uint64_t atomic_fetch_or(uint64_t *p, uint64_t v)
{
    return __hip_atomic_fetch_or(p, v, __ATOMIC_RELAXED, SHMEMX_AGENT);
}
__device__ __forceinline__ uint64_t atomic_compare_swap(uint64_t *p, uint64_t cond, uint64_t v)
{
    __hip_atomic_compare_exchange_strong(p, &cond, v, __ATOMIC_RELAXED, __ATOMIC_RELAXED, SHMEMX_AGENT);
    return cond;  // the previous value, whether or not the swap happened
}
__device__ __forceinline__ uint64_t atomic_fetch(const uint64_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, SHMEMX_AGENT);
}

// ---------------------------------------------------------------------------
// Ordering.  quiet: the calling wave's earlier puts / AMOs are complete and
// visible device-wide (wait for outstanding stores, write this XCD's L2 back).
// fence: earlier puts ordered before later ones; on one GPU that is the same
// release, so both map to it.  acquire: drop stale lines before reading what
// another PE put (needed after a barrier or after seeing a signal).
__device__ __forceinline__ void quiet() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent"); }
__device__ __forceinline__ void fence() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent"); }
__device__ __forceinline__ void acquire() { __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent"); }

// The device-scope release and acquire around a barrier are cache maintenance
// on the die's L2 (write back dirty lines / drop stale ones), so one wave per
// workgroup performs them: every wave first completes its own stores
// (workgroup-scope release) and meets the others; wave 0 then releases at
// device scope, synchronises with the other workgroups and acquires at device
// scope -- the L1 it invalidates is the one all waves of the workgroup share --
// before the workgroup continues.
__device__ __forceinline__ void wg_release()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
}
__device__ __forceinline__ void wg_acquire()
{
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// One arrival at a sense-reversing barrier word pair (thread 0 of a workgroup).
// Returns true for the last of `n` arrivals, which must call barrier_open when
// it is ready to let the others go; everybody else returns after the wait.
// Waits are bounded (about a second); once any wait of a launch has timed out
// the fault word is set and every later wait gives up at once, so a broken
// launch still drains quickly.
__device__ __forceinline__ bool barrier_arrive(const Ctx &c, uint64_t *count, uint64_t *gen, uint32_t n,
                                               uint64_t *my_gen)
{
    // All atomics here are relaxed: the caller's quiet() before and acquire() after are the
    // fences.  (An acquire on every poll would invalidate the die's L2 once per poll.)
    // The generation must be read BEFORE the arrival is counted (counted first, the last arriver could open the
    // barrier before this read, which would then see the new generation and wait for a release that has
    // already happened).  The two are relaxed atomics on different addresses, which neither the compiler nor
    // the memory system keeps in order by themselves: the empty asm consumes the loaded value, so the wave has
    // the generation in a register (the load has returned) before the add can be issued.
    uint64_t g = __hip_atomic_load(gen, __ATOMIC_RELAXED, SHMEMX_AGENT);
    asm volatile("" : "+v"(g) : : "memory");
    *my_gen = g;
    const uint64_t a = __hip_atomic_fetch_add(count, 1ull, __ATOMIC_RELAXED, SHMEMX_AGENT);
    if (a == n - 1) {
        __hip_atomic_store(count, 0ull, __ATOMIC_RELAXED, SHMEMX_AGENT);
        return true;
    }
    uint32_t spins = 0;
    while (__hip_atomic_load(gen, __ATOMIC_RELAXED, SHMEMX_AGENT) == g) {
        if (timed_out(c, spins)) break;
        __builtin_amdgcn_s_sleep(2);
        if (++spins > SPIN_LIMIT) { report(c, DEV_ERR_BARRIER_TIMEOUT, blockIdx.x); break; }
    }
    return false;
}
// The last arriver has read every other arrival; the fence makes what they released part of
// what the waiters acquire when they see the new generation.
__device__ __forceinline__ void barrier_open(uint64_t *gen, uint64_t my_gen)
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "agent");
    __hip_atomic_store(gen, my_gen + 1, __ATOMIC_RELAXED, SHMEMX_AGENT);
}

// Team barrier: the workgroups of one PE.  Implies a PE-wide quiet before and
// an acquire after.  Every participating workgroup must be resident (the host checks the
// grid against the occupancy limit and uses a cooperative launch).
__device__ __forceinline__ void team_barrier(const Ctx &c, uint32_t pe, uint32_t wgs_per_pe)
{
    wg_release();
    if (threadIdx.x == 0) {
        quiet();
        if (wgs_per_pe > 1) {   // a one-workgroup team has nobody else to meet
            uint64_t *w = &c.scratch[W_PE_BASE + pe * W_PE_WORDS], g;
            if (barrier_arrive(c, w, w + 16, wgs_per_pe, &g)) barrier_open(w + 16, g);
            acquire();
        }
    }
    wg_acquire();
}

// World barrier (barrier_all): quiet by every wave, then the workgroups meet.  Up to
// FLAT_BARRIER_WGS workgroups in the launch arrive on the world words directly: arrivals on one
// address serialise at about 12 ns each, which for a few dozen is less than a second round trip.
// Larger launches take two stages so that no word is hammered by more than max(wgs_per_pe, npes)
// workgroups -- the workgroups of a team meet on the team's words, the last one of each team
// meets the other teams on the world words and then releases its team.
constexpr uint32_t FLAT_BARRIER_WGS = 256;

__device__ __forceinline__ void barrier_all(const Ctx &c, uint32_t pe, uint32_t wgs_per_pe)
{
    wg_release();
    if (threadIdx.x == 0) {
        quiet();
        const uint32_t total = (uint32_t)c.npes * wgs_per_pe;
        uint64_t *t = &c.scratch[W_PE_BASE + pe * W_PE_WORDS + 32], tg, wg_;
        if (total <= FLAT_BARRIER_WGS) {
            if (barrier_arrive(c, &c.scratch[W_BAR_COUNT], &c.scratch[W_BAR_GEN], total, &wg_))
                barrier_open(&c.scratch[W_BAR_GEN], wg_);
        } else if (barrier_arrive(c, t, t + 16, wgs_per_pe, &tg)) {
            if (barrier_arrive(c, &c.scratch[W_BAR_COUNT], &c.scratch[W_BAR_GEN], (uint32_t)c.npes, &wg_))
                barrier_open(&c.scratch[W_BAR_GEN], wg_);
            barrier_open(t + 16, tg);
        }
        acquire();
    }
    wg_acquire();
}

// Barrier over a team of PEs -- the members start, start + stride, ... (size of them; the barrier session
// of Listing 1 takes a team, OpenSHMEM calls it an active set): quiet by every wave of the members, the
// workgroups of a member meet on that PE's words, the last one of each member meets the other members on
// the team's own words (the copy on the team's first PE) and then releases its PE.  Every workgroup of
// every member must call it; the others are not involved and may be in a barrier of their own team.
struct PeTeam {
    uint32_t start, stride, size;
    uint32_t pad;
    uint64_t words_off;   // symmetric, 256 bytes: arrivals at +0, generation at +128
    __device__ __forceinline__ bool has(uint32_t pe) const
    {
        return pe >= start && (pe - start) % stride == 0 && (pe - start) / stride < size;
    }
    __device__ __forceinline__ uint32_t index_of(uint32_t pe) const { return (pe - start) / stride; }
    __device__ __forceinline__ uint32_t member(uint32_t i) const { return start + i * stride; }
};

__device__ __forceinline__ void pe_team_sync(const Ctx &c, const PeTeam &t, uint32_t pe, uint32_t wgs_per_pe)
{
    wg_release();
    if (threadIdx.x == 0) {
        quiet();
        uint64_t *mine = &c.scratch[W_PE_BASE + pe * W_PE_WORDS + 32], mg = 0, tg;   // a PE is in one barrier at a time
        if (wgs_per_pe == 1 || barrier_arrive(c, mine, mine + 16, wgs_per_pe, &mg)) {
            uint64_t *w = (uint64_t *)ptr(c, t.words_off, t.start);
            if (t.size > 1 && barrier_arrive(c, w, w + 16, t.size, &tg)) barrier_open(w + 16, tg);
            if (wgs_per_pe > 1) barrier_open(mine + 16, mg);
        }
        acquire();
    }
    wg_acquire();
}

// ---------------------------------------------------------------------------
// Contiguous copy by `size` cooperating lanes (rank in [0, size)).  Lane r
// moves 16-byte vectors r, r+size, ... so that a wavefront's access covers
// 1 KiB of consecutive bytes; four loads are in flight per lane before the
// first store.  The widest unit the two addresses share (16/8/4/1 bytes) is
// used; head and tail bytes are peeled.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// A store that is WRITTEN THROUGH to memory (the system-coherent form of the store instruction): it leaves no
// dirty line in the die's L2.  For data that a device-scope release is about to make visible -- a put that a
// signal, a quiet or a barrier follows: that release writes back whatever the L2 holds dirty, which under load
// takes microseconds, and with the data written through it finds next to nothing.  (Data whose completion is a
// kernel boundary keeps streaming stores, which are faster in bulk.)
__device__ __forceinline__ void store_through(u32x4 v, u32x4 *d)
{
    // (the idle cycle: the instruction that follows a store of more than 8 bytes must not write the registers that
    // hold its data, which the compiler sees to for its own stores and cannot for this one)
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 0" : : "v"(d), "v"(v) : "memory");
}
__device__ __forceinline__ void store_through(u32x2 v, u32x2 *d)
{
    asm volatile("global_store_dwordx2 %0, %1, off sc0 sc1" : : "v"(d), "v"(v) : "memory");
}
__device__ __forceinline__ void store_through(uint32_t v, uint32_t *d)
{
    asm volatile("global_store_dword %0, %1, off sc0 sc1" : : "v"(d), "v"(v) : "memory");
}
__device__ __forceinline__ void store_through(uint8_t v, uint8_t *d)
{
    asm volatile("global_store_byte %0, %1, off sc0 sc1" : : "v"(d), "v"((uint32_t)v) : "memory");
}
template <bool THROUGH, typename V>
__device__ __forceinline__ void copy_store(V v, V *d)
{
    if (THROUGH) store_through(v, d); else __builtin_nontemporal_store(v, d);
}

template <bool THROUGH, typename V>
__device__ __forceinline__ void copy_units(V *__restrict__ d, const V *__restrict__ s, size_t nv,
                                           size_t rank, size_t size)
{
    size_t i = rank;
    for (; i + 3 * size < nv; i += 4 * size) {
        V a = __builtin_nontemporal_load(s + i);
        V b = __builtin_nontemporal_load(s + i + size);
        V e = __builtin_nontemporal_load(s + i + 2 * size);
        V f = __builtin_nontemporal_load(s + i + 3 * size);
        copy_store<THROUGH>(a, d + i);
        copy_store<THROUGH>(b, d + i + size);
        copy_store<THROUGH>(e, d + i + 2 * size);
        copy_store<THROUGH>(f, d + i + 3 * size);
    }
    // up to three units are left for this lane: all loads first, then the stores
    const bool p0 = i < nv, p1 = i + size < nv, p2 = i + 2 * size < nv;
    V a, b, e;
    if (p0) a = __builtin_nontemporal_load(s + i);
    if (p1) b = __builtin_nontemporal_load(s + i + size);
    if (p2) e = __builtin_nontemporal_load(s + i + 2 * size);
    if (p0) copy_store<THROUGH>(a, d + i);
    if (p1) copy_store<THROUGH>(b, d + i + size);
    if (p2) copy_store<THROUGH>(e, d + i + 2 * size);
}

// THROUGH: the destination is written through (see store_through).
template <bool THROUGH = false>
__device__ __forceinline__ void copy(uint8_t *__restrict__ dst, const uint8_t *__restrict__ src, size_t n,
                                     size_t rank, size_t size)
{
    if (n == 0) return;
    const uintptr_t diff = (uintptr_t)dst ^ (uintptr_t)src;
    const size_t unit = (diff & 15) == 0 ? 16 : (diff & 7) == 0 ? 8 : (diff & 3) == 0 ? 4 : 1;
    size_t head = (size_t)(-(uintptr_t)dst) & (unit - 1);
    if (head > n) head = n;
    for (size_t j = rank; j < head; j += size) copy_store<THROUGH>(src[j], dst + j);
    const size_t body = (n - head) / unit;
    uint8_t *d = dst + head;
    const uint8_t *s = src + head;
    if (unit == 16) copy_units<THROUGH>((u32x4 *)d, (const u32x4 *)s, body, rank, size);
    else if (unit == 8) copy_units<THROUGH>((u32x2 *)d, (const u32x2 *)s, body, rank, size);
    else if (unit == 4) copy_units<THROUGH>((uint32_t *)d, (const uint32_t *)s, body, rank, size);
    else copy_units<THROUGH>(d, s, body, rank, size);
    for (size_t j = head + body * unit + rank; j < n; j += size) copy_store<THROUGH>(src[j], dst + j);
}

// A large contiguous copy with 16-byte aligned ends by `waves` cooperating waves (this one is number
// `my`): the leading multiple of 4 KiB streams through a software-pipelined loop over two register sets
// (wave-tasks of 4 KiB dealt round robin, a wave's next task requested before its current one is stored);
// wave 0 moves the rest through the generic copy.
__device__ __forceinline__ void copy_stream(uint8_t *__restrict__ dst, const uint8_t *__restrict__ src, size_t n,
                                            uint64_t my, uint64_t waves, uint32_t lane)
{
    constexpr int VPL = 4;
    constexpr uint64_t TASK = 1024ull * VPL;
    const uint64_t tasks = n / TASK;
    if (my == 0 && n > tasks * TASK) copy(dst + tasks * TASK, src + tasks * TASK, n - tasks * TASK, lane, 64);
    if (my >= tasks) return;
    uint64_t left = (tasks - 1 - my) / waves;            // tasks of this wave after its first
    const uint32_t lane_off = lane * 16;
    uint64_t t = my;
    u32x4 va[VPL], vb[VPL];
    const uint8_t *s = src + t * TASK;
    uint8_t *da = dst + t * TASK, *db = nullptr;
#pragma unroll
    for (int j = 0; j < VPL; ++j) va[j] = __builtin_nontemporal_load((const u32x4 *)(s + lane_off) + 64 * j);
    for (;;) {
        if (left == 0) {
#pragma unroll
            for (int j = 0; j < VPL; ++j) __builtin_nontemporal_store(va[j], (u32x4 *)(da + lane_off) + 64 * j);
            break;
        }
        t += waves; s = src + t * TASK; db = dst + t * TASK;
#pragma unroll
        for (int j = 0; j < VPL; ++j) vb[j] = __builtin_nontemporal_load((const u32x4 *)(s + lane_off) + 64 * j);
#pragma unroll
        for (int j = 0; j < VPL; ++j) __builtin_nontemporal_store(va[j], (u32x4 *)(da + lane_off) + 64 * j);
        if (left == 1) {
#pragma unroll
            for (int j = 0; j < VPL; ++j) __builtin_nontemporal_store(vb[j], (u32x4 *)(db + lane_off) + 64 * j);
            break;
        }
        t += waves; s = src + t * TASK; da = dst + t * TASK;
#pragma unroll
        for (int j = 0; j < VPL; ++j) va[j] = __builtin_nontemporal_load((const u32x4 *)(s + lane_off) + 64 * j);
#pragma unroll
        for (int j = 0; j < VPL; ++j) __builtin_nontemporal_store(vb[j], (u32x4 *)(db + lane_off) + 64 * j);
        left -= 2;
    }
}

constexpr size_t PUT_THROUGH_BYTES = 4096;
// put / get are the same copy with the remote side as destination / source.  (They stay on the generic
// copy: pulling the streaming loop into the latency kernels cost 0.4 us per ping-pong round trip.)
// (Sec. III-A one-sided semantics; Table II put_nbi / get).
__device__ __forceinline__ void put(const Ctx &c, uint64_t dst_off, const uint8_t *src, size_t n, uint32_t pe,
                                    size_t rank, size_t size)
{
    // a small put is written through: what follows it is a quiet, a signal or a barrier, whose release then has
    // nothing of it left to write back (ping-pong of 8 B to 4 KiB: 2.7-2.8 -> 2.3-2.5 us per round trip); larger
    // ones keep streaming stores, which carry far more per workgroup (64 KiB: 6.1 us against 9.7)
    if (n <= PUT_THROUGH_BYTES) copy<true>(ptr(c, dst_off, pe), src, n, rank, size);
    else copy<false>(ptr(c, dst_off, pe), src, n, rank, size);
}
__device__ __forceinline__ void get(const Ctx &c, uint8_t *dst, uint64_t src_off, size_t n, uint32_t pe,
                                    size_t rank, size_t size)
{
    copy(dst, ptr(c, src_off, pe), n, rank, size);
}

// ---------------------------------------------------------------------------
// Strided copy: d[i * ds] = s[i * ss], i < nelems, strides in elements.
// Lane r takes elements r, r + size, ... (lane-major), so one wave access spans
// 64 * pitch consecutive bytes on a strided side -- for small pitches a handful
// of cache lines, each fully used by neighbouring lanes -- and 64 consecutive
// elements on a unit-stride side.  SIF elements are in flight per lane before
// the first store.  Only the named elements are written: the gaps of a strided
// destination may belong to somebody else's concurrent iput.
constexpr int SIF = 8;

template <typename T>
__device__ __forceinline__ void strided_t(T *__restrict__ d, const T *__restrict__ s, int64_t ds, int64_t ss,
                                          size_t nelems, size_t rank, size_t size)
{
    size_t i = rank;
    for (; i + (SIF - 1) * size < nelems; i += SIF * size) {
        T v[SIF];
#pragma unroll
        for (int k = 0; k < SIF; ++k) v[k] = __builtin_nontemporal_load(s + (i + k * size) * ss);
#pragma unroll
        for (int k = 0; k < SIF; ++k) __builtin_nontemporal_store(v[k], d + (i + k * size) * ds);
    }
    for (; i < nelems; i += size) d[i * ds] = s[i * ss];
}

__device__ __forceinline__ void strided(uint8_t *d, const uint8_t *s, int64_t ds, int64_t ss, size_t nelems,
                                        uint32_t elem_bytes, size_t rank, size_t size)
{
    switch (elem_bytes) {
    case 8: strided_t((uint64_t *)d, (const uint64_t *)s, ds, ss, nelems, rank, size); break;
    case 4: strided_t((uint32_t *)d, (const uint32_t *)s, ds, ss, nelems, rank, size); break;
    case 2: strided_t((uint16_t *)d, (const uint16_t *)s, ds, ss, nelems, rank, size); break;
    default: strided_t(d, s, ds, ss, nelems, rank, size); break;
    }
}

// ---------------------------------------------------------------------------
// Wavefront helpers (64 lanes).
__device__ __forceinline__ uint32_t lane_id() { return __lane_id(); }
__device__ __forceinline__ uint64_t ballot(bool p) { return __ballot(p); }
__device__ __forceinline__ uint32_t rank_in(uint64_t mask)  // set bits of mask below this lane
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}
__device__ __forceinline__ uint32_t bcast32(uint32_t v, uint32_t lane) { return __builtin_amdgcn_readlane(v, lane); }
__device__ __forceinline__ uint64_t bcast64(uint64_t v, uint32_t lane)
{
    uint32_t lo = __builtin_amdgcn_readlane((uint32_t)v, lane);
    uint32_t hi = __builtin_amdgcn_readlane((uint32_t)(v >> 32), lane);
    return ((uint64_t)hi << 32) | lo;
}

}  // namespace shmemx

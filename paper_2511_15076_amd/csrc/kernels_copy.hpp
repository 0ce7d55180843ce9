// put / get / iput / iget kernels: stand-alone ops, the descriptor-table
// executor and the bandwidth-sweep cell.
#pragma once
#include "../../include/mi_shmem.h"
#include "../../include/mi_shmemx.hpp"

namespace shmemx {

// One contiguous put or get: the whole grid is the initiator's team.
__global__ __launch_bounds__(256) void k_copy(uint8_t *__restrict__ dst, const uint8_t *__restrict__ src, size_t n)
{
    copy(dst, src, n, (size_t)blockIdx.x * blockDim.x + threadIdx.x, (size_t)gridDim.x * blockDim.x);
}

// One strided iput or iget.
__global__ __launch_bounds__(256) void k_strided(uint8_t *__restrict__ dst, const uint8_t *__restrict__ src,
                                                 int64_t ds, int64_t ss, size_t nelems, uint32_t eb)
{
    strided(dst, src, ds, ss, nelems, eb, (size_t)blockIdx.x * blockDim.x + threadIdx.x,
            (size_t)gridDim.x * blockDim.x);
}

// ---------------------------------------------------------------------------
// Descriptor-table executor (one persistent launch).  PE team p = workgroups
// [p * wgs_per_pe, (p+1) * wgs_per_pe).  Every wave of a team walks the
// window's descriptors (uniform loads) and picks its share of the team's ops:
// small ops go round-robin to single waves (wave-cooperative put / get), ops
// above BIG_OP bytes are done by all waves of the team together.  At a window
// end every wave performs quiet and the teams meet in the world barrier.
// STREAM selects how a large aligned put / get is moved: through the pipelined
// streaming copy (teams of many workgroups, where it is worth 6 % of bandwidth)
// or through the generic copy, which keeps the kernel a third of the size -- the
// variant for small teams, whose tables of small ops are latency-bound.
// ---------------------------------------------------------------------------
constexpr uint64_t BIG_OP = 64 * 1024;

__device__ __forceinline__ bool desc_valid(const Ctx &c, const shmem_op_desc &d)
{
    if (d.pe >= (uint32_t)c.npes) return false;
    if (d.kind == SHMEM_OP_PUT || d.kind == SHMEM_OP_GET)
        return d.local_off <= c.seg && d.count <= c.seg - d.local_off && d.sym_off <= c.seg &&
               d.count <= c.seg - d.sym_off;
    if (d.kind == SHMEM_OP_IPUT || d.kind == SHMEM_OP_IGET) {
        const uint32_t eb = d.elem_bytes;
        if (eb != 1 && eb != 2 && eb != 4 && eb != 8) return false;
        if (d.local_stride < 1 || d.sym_stride < 1) return false;
        if (d.local_off % eb || d.sym_off % eb) return false;
        if (d.count == 0) return d.local_off <= c.seg && d.sym_off <= c.seg;
        // spans, with overflow guarded by bounding each factor by the segment size
        // (a stride only matters from the second element on; bounding the factors keeps the products in 128 bits)
        if (d.count > c.seg || (d.count > 1 && ((uint64_t)d.local_stride > c.seg || (uint64_t)d.sym_stride > c.seg))) return false;
        const unsigned __int128 ls = (unsigned __int128)(d.count - 1) * (uint64_t)d.local_stride * eb + eb;
        const unsigned __int128 ss = (unsigned __int128)(d.count - 1) * (uint64_t)d.sym_stride * eb + eb;
        return d.local_off <= c.seg && ls <= c.seg - d.local_off && d.sym_off <= c.seg && ss <= c.seg - d.sym_off;
    }
    return false;
}

// THROUGH: contiguous destinations are written through to memory (see store_through; the operations of a table
// are not: with a few KiB per window there is little for the window's release to write back, and the stores'
// own completion is slower -- configuration 1 ran at 6.4 instead of 5.5 us per window with it).
template <bool THROUGH>
__device__ __forceinline__ void desc_exec(const Ctx &c, const shmem_op_desc &d, size_t rank, size_t size)
{
    uint8_t *local = ptr(c, d.local_off, d.pe_self);
    uint8_t *remote = ptr(c, d.sym_off, d.pe);
    switch (d.kind) {
    case SHMEM_OP_PUT: copy<THROUGH>(remote, local, d.count, rank, size); break;
    case SHMEM_OP_GET: copy<THROUGH>(local, remote, d.count, rank, size); break;
    case SHMEM_OP_IPUT: strided(remote, local, d.sym_stride, d.local_stride, d.count, d.elem_bytes, rank, size); break;
    case SHMEM_OP_IGET: strided(local, remote, d.local_stride, d.sym_stride, d.count, d.elem_bytes, rank, size); break;
    default: break;
    }
}

template <bool STREAM>
__global__ __launch_bounds__(256, 4) void k_op_batch(Ctx c, const shmem_op_desc *__restrict__ ops, size_t n,
                                                  size_t quiet_every, int wgs_per_pe)
{
    const uint32_t pe = blockIdx.x / (uint32_t)wgs_per_pe;
    const uint32_t wg = blockIdx.x % (uint32_t)wgs_per_pe;
    const uint32_t lane = threadIdx.x & 63, waves_per_wg = blockDim.x >> 6;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t team_waves = (uint32_t)wgs_per_pe * waves_per_wg;
    const uint32_t my_wave = wg * waves_per_wg + wave;
    const size_t window = quiet_every ? quiet_every : n;
    // 64 descriptors at a time: lane j reads descriptor j (one coalesced 4 KiB read), a ballot finds
    // this PE's ones, and their fields are broadcast from the lane that holds them.  The next batch
    // is requested before the current one is executed -- also across a window end, so the read of the
    // next window's first descriptors travels during the barrier (the table is read-only).
    auto load = [&](size_t i0, size_t e) {
        shmem_op_desc d;
        d.kind = ~0u; d.pe_self = ~0u; d.pe = 0; d.elem_bytes = 0; d.local_off = d.sym_off = d.count = 0;
        d.local_stride = d.sym_stride = 0; d.value = 0;
        if (i0 + lane < e) d = ops[i0 + lane];
        return d;
    };
    size_t b = 0, e = window < n ? window : n, i0 = 0;
    shmem_op_desc d = n ? load(0, e) : shmem_op_desc();
    uint32_t mine = 0;  // small ops of this PE seen so far in the window
    while (i0 < n) {
        // position of the batch after this one
        const bool last_of_window = i0 + 64 >= e;
        const size_t nb = last_of_window ? e : b, ni0 = last_of_window ? e : i0 + 64;
        const size_t ne = last_of_window ? (e + window < n ? e + window : n) : e;
        shmem_op_desc dn = load(ni0, ni0 < n ? ne : ni0);                      // nothing to load past the end
        {
            const bool have = i0 + lane < e;
            if (have && d.pe_self >= (uint32_t)c.npes && blockIdx.x == 0 && wave == 0) report(c, DEV_ERR_BAD_OP, i0 + lane);
            const bool ok = have && d.pe_self == pe && desc_valid(c, d);
            if (have && d.pe_self == pe && !ok && wg == 0 && wave == 0) report(c, DEV_ERR_BAD_OP, i0 + lane);
            // Which of the PE's ops this wave executes is settled for all 64 descriptors at once: large
            // ops are everybody's, small op number k of the window (a ballot and a prefix count give k)
            // belongs to wave k mod team_waves.  The wave then walks only its own ops: walking all of the
            // PE's ops and skipping the others' cost about 100 instructions each, several microseconds
            // per window for a wave that has the SIMD to itself.
            const uint64_t bytes_l = (d.kind <= SHMEM_OP_GET) ? d.count : d.count * d.elem_bytes;
            const bool big = ok && bytes_l > BIG_OP;
            const uint64_t small_mask = ballot(ok && !big);
            const uint32_t ordinal = mine + rank_in(small_mask);
            uint64_t todo = ballot(big || (ok && !big && ordinal % team_waves == my_wave));
            mine += (uint32_t)__builtin_popcountll(small_mask);
            while (todo) {
                const uint32_t j = (uint32_t)__builtin_ctzll(todo);
                todo &= todo - 1;
                shmem_op_desc u;                      // descriptor j, now uniform across the wave
                u.kind = bcast32(d.kind, j); u.pe_self = pe; u.pe = bcast32(d.pe, j);
                u.elem_bytes = bcast32(d.elem_bytes, j);
                u.local_off = bcast64(d.local_off, j); u.sym_off = bcast64(d.sym_off, j);
                u.count = bcast64(d.count, j);
                u.local_stride = (int64_t)bcast64((uint64_t)d.local_stride, j);
                u.sym_stride = (int64_t)bcast64((uint64_t)d.sym_stride, j);
                const uint64_t bytes = (u.kind <= SHMEM_OP_GET) ? u.count : u.count * u.elem_bytes;
                if (bytes > BIG_OP) {
                    uint8_t *local = ptr(c, u.local_off, pe), *remote = ptr(c, u.sym_off, u.pe);
                    if (STREAM && u.kind <= SHMEM_OP_GET && (((uintptr_t)local | (uintptr_t)remote) & 15) == 0) {
                        if (u.kind == SHMEM_OP_PUT) copy_stream(remote, local, u.count, my_wave, team_waves, lane);
                        else copy_stream(local, remote, u.count, my_wave, team_waves, lane);
                    } else {
                        desc_exec<false>(c, u, (size_t)my_wave * 64 + lane, (size_t)team_waves * 64);
                    }
                } else {
                    desc_exec<false>(c, u, lane, 64);
                }
            }
        }
        if (last_of_window) {
            barrier_all(c, pe, (uint32_t)wgs_per_pe);  // quiet by every wave, then all teams synchronise
            mine = 0;
        }
        d = dn; b = nb; i0 = ni0; e = ne;
    }
}

// ---------------------------------------------------------------------------
// Bandwidth-sweep cell.  All ops of a PE are independent, so the team's waves
// share the flattened list of (op, chunk) tasks: a chunk is CHUNK_VECS 16-byte
// vectors per lane (4 KiB per wave for contiguous ops, 2048 elements for
// strided ones).  Neighbouring waves take neighbouring chunks, so a workgroup
// streams 16 KiB of consecutive bytes per step.
struct SweepArgs {
    int kind;
    uint64_t remote_off, local_off;
    uint64_t count;
    uint32_t elem_bytes;
    int64_t remote_stride, local_stride;
    uint64_t remote_slot, local_slot, nslots;
    uint32_t ops_per_pe, wgs_per_pe;
};

constexpr uint64_t CHUNK_BYTES = 4096;  // per wave-task, contiguous ops
constexpr uint64_t CHUNK_ELEMS = 2048;  // per wave-task, strided ops
constexpr uint64_t SMALL_MSG = 512;     // contiguous messages up to this size (twice that with 16-byte alignment: what one
                                        // wave instruction covers) are packed into sub-wave groups

// Contiguous 16-byte aligned messages of at least 1 KiB (the bandwidth cells), their leading multiple of
// 1 KiB: every
// wave-task is VPL full 16-byte vectors per lane, so nothing is predicated, and the loop is software-
// pipelined over two register sets: the loads of a wave's next task are issued before the stores of
// its current one, which keeps reads in flight behind the writes.  (Predicated or conditional loads
// inside the loop would make the compiler wait for every outstanding access before each store.)
template <int VPL>
__device__ __forceinline__ void sweep_pipelined(const SweepArgs &a, uint64_t first, uint64_t body, uint8_t *lbase, uint8_t *rbase,
                                                uint64_t my_wave, uint64_t team_waves, uint32_t lane)
{
    constexpr uint64_t TASK_VECS = 64 * VPL;
    const uint64_t chunks = body / (TASK_VECS * 16);   // bytes [first, first + body) of every message are moved here
    const uint64_t tasks = chunks * a.ops_per_pe;
    if (my_wave >= tasks) return;
    // task t = (op, chunk) with slot = op % nslots; the walk t -> t + team_waves needs no division
    const uint64_t step_ch = team_waves % chunks, step_slot = (team_waves / chunks) % a.nslots;
    uint64_t ch = my_wave % chunks, slot = (my_wave / chunks) % a.nslots;
    uint64_t left = (tasks - 1 - my_wave) / team_waves;  // tasks of this wave after its first
    const bool is_put = a.kind == SHMEM_OP_PUT;
    // wave-uniform bases plus one constant per-lane byte offset: the addresses live in scalar registers
    const uint8_t *const sbase = (is_put ? lbase : rbase) + first;
    uint8_t *const dbase = (is_put ? rbase : lbase) + first;
    const uint64_t sslot = is_put ? a.local_slot : a.remote_slot, dslot = is_put ? a.remote_slot : a.local_slot;
    const uint32_t lane_off = lane * 16;
    auto locate = [&](const uint8_t *&src, uint8_t *&dst) {
        src = sbase + slot * sslot + ch * (TASK_VECS * 16);
        dst = dbase + slot * dslot + ch * (TASK_VECS * 16);
    };
    auto advance = [&]() {
        ch += step_ch;
        slot += step_slot;
        if (ch >= chunks) { ch -= chunks; slot += 1; }
        if (slot >= a.nslots) slot -= a.nslots;
    };
    auto load = [&](u32x4 (&v)[VPL], const uint8_t *src) {
#pragma unroll
        for (int j = 0; j < VPL; ++j) v[j] = __builtin_nontemporal_load((const u32x4 *)(src + lane_off) + 64 * j);
    };
    auto store = [&](const u32x4 (&v)[VPL], uint8_t *dst) {
#pragma unroll
        for (int j = 0; j < VPL; ++j) __builtin_nontemporal_store(v[j], (u32x4 *)(dst + lane_off) + 64 * j);
    };
    u32x4 va[VPL], vb[VPL];
    const uint8_t *src;
    uint8_t *da, *db;
    locate(src, da);
    load(va, src);
    for (;;) {
        if (left == 0) { store(va, da); break; }
        advance();
        locate(src, db);
        load(vb, src);
        store(va, da);
        if (left == 1) { store(vb, db); break; }
        advance();
        locate(src, da);
        load(va, src);
        store(vb, db);
        left -= 2;
    }
}

// The same pipeline for messages of 4 KiB and more whose length is a multiple of 16 bytes but not of
// 4 KiB: the last task of every message is short.  Nothing is predicated here either -- a lane whose
// vector lies beyond the end of the message moves the message's LAST vector again (same bytes to the same
// place; the lanes of such an instruction share one address, so it is one request) -- which keeps the
// number of accesses per task fixed and the waits partial.  One pass moves the whole message, including a
// remainder under 1 KiB such as the 16 metadata bytes of a 14,352-byte MoE message.
__device__ __forceinline__ void sweep_pipelined_ragged(const SweepArgs &a, uint8_t *lbase, uint8_t *rbase, uint64_t my_wave,
                                                       uint64_t team_waves, uint32_t lane)
{
    constexpr int VPL = 4;
    constexpr uint64_t TASK_VECS = 64 * VPL, TASK_BYTES = TASK_VECS * 16;
    const uint64_t chunks = (a.count + TASK_BYTES - 1) / TASK_BYTES;
    const uint32_t last_vecs = (uint32_t)((a.count - (chunks - 1) * TASK_BYTES) / 16);   // 1 .. TASK_VECS
    const uint64_t tasks = chunks * a.ops_per_pe;
    if (my_wave >= tasks) return;
    const uint64_t step_ch = team_waves % chunks, step_slot = (team_waves / chunks) % a.nslots;
    uint64_t ch = my_wave % chunks, slot = (my_wave / chunks) % a.nslots;
    uint64_t left = (tasks - 1 - my_wave) / team_waves;
    const bool is_put = a.kind == SHMEM_OP_PUT;
    const uint8_t *const sbase = is_put ? lbase : rbase;
    uint8_t *const dbase = is_put ? rbase : lbase;
    const uint64_t sslot = is_put ? a.local_slot : a.remote_slot, dslot = is_put ? a.remote_slot : a.local_slot;
    auto locate = [&](const uint8_t *&src, uint8_t *&dst, uint32_t &nv) {
        src = sbase + slot * sslot + ch * TASK_BYTES;
        dst = dbase + slot * dslot + ch * TASK_BYTES;
        nv = ch == chunks - 1 ? last_vecs : (uint32_t)TASK_VECS;
    };
    auto advance = [&]() {
        ch += step_ch;
        slot += step_slot;
        if (ch >= chunks) { ch -= chunks; slot += 1; }
        if (slot >= a.nslots) slot -= a.nslots;
    };
    auto load = [&](u32x4 (&v)[VPL], const uint8_t *src, uint32_t nv) {
#pragma unroll
        for (int j = 0; j < VPL; ++j) v[j] = __builtin_nontemporal_load((const u32x4 *)src + min(lane + 64u * j, nv - 1));
    };
    auto store = [&](const u32x4 (&v)[VPL], uint8_t *dst, uint32_t nv) {
#pragma unroll
        for (int j = 0; j < VPL; ++j) __builtin_nontemporal_store(v[j], (u32x4 *)dst + min(lane + 64u * j, nv - 1));
    };
    u32x4 va[VPL], vb[VPL];
    const uint8_t *src;
    uint8_t *da, *db;
    uint32_t na, nb;
    locate(src, da, na);
    load(va, src, na);
    for (;;) {
        if (left == 0) { store(va, da, na); break; }
        advance();
        locate(src, db, nb);
        load(vb, src, nb);
        store(va, da, na);
        if (left == 1) { store(vb, db, nb); break; }
        advance();
        locate(src, da, na);
        load(va, src, na);
        store(vb, db, nb);
        left -= 2;
    }
}

// One large contiguous put or get with 16-byte aligned ends: the whole grid is the initiator's team.
__global__ __launch_bounds__(256) void k_copy_stream(uint8_t *__restrict__ dst, const uint8_t *__restrict__ src, size_t n)
{
    const uint32_t lane = threadIdx.x & 63, waves_per_wg = blockDim.x >> 6;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    copy_stream(dst, src, n, (uint64_t)blockIdx.x * waves_per_wg + wave, (uint64_t)gridDim.x * waves_per_wg, lane);
}

// Small messages (up to 64 vectors of 8 or 16 bytes): a sub-group of lanes, one vector V per
// lane, moves one message, so a wave instruction carries 64 / group messages; sets of four such rounds
// alternate between two register sets, the loads of the next set going out before the stores of the
// current one (with one round at a time a wave had 512 bytes in flight and the small sizes were
// latency-bound).
template <typename V>
__device__ __forceinline__ void sweep_small(const SweepArgs &a, uint8_t *lbase, uint8_t *rbase, uint64_t my_wave,
                                            uint64_t team_waves, uint32_t lane)
{
    constexpr uint32_t W = sizeof(V);
    constexpr int U = 4;                                   // rounds per register set; two sets alternate
    uint32_t group = 1;
    while (group * W < a.count) group <<= 1;
    const uint32_t per_wave = 64 / group, sub = lane / group;
    // Nothing is predicated (a load under a condition makes every later wait a wait for everything in
    // flight, the stores included): a lane beyond the end of its message moves the message's last vector
    // again, and a lane beyond the last operation moves the last operation again -- the same bytes to the
    // same place, harmless whoever does it.  Whole sets of U rounds go through the two-set pipeline; the
    // up to U - 1 rounds that are left are moved one at a time (repeating rounds to fill a set made the
    // smallest messages several times slower where a wave has only a round or two).
    const uint32_t nvec = (uint32_t)(a.count / W);         // the host sends count as a multiple of W, at least W
    const uint32_t j = min(lane % group, nvec - 1);
    const uint64_t last_op = a.ops_per_pe - 1;
    const uint64_t rounds_all = (a.ops_per_pe + per_wave - 1) / per_wave;      // rounds of the whole team
    if (my_wave >= rounds_all) return;
    const uint64_t mine = (rounds_all - 1 - my_wave) / team_waves + 1;          // rounds of this wave
    uint64_t sets = mine / U;
    const uint32_t rest = (uint32_t)(mine % U);
    const bool is_put = a.kind == SHMEM_OP_PUT;
    const uint8_t *const sbase = is_put ? lbase : rbase;
    uint8_t *const dbase = is_put ? rbase : lbase;
    const uint64_t sslot = is_put ? a.local_slot : a.remote_slot, dslot = is_put ? a.remote_slot : a.local_slot;
    uint64_t t = my_wave;                                  // first round of the next set to load
    auto load = [&](V (&v)[U], V *(&dst)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t op_ = (t + (uint64_t)u * team_waves) * per_wave + sub;
            const uint64_t op = op_ < last_op ? op_ : last_op;
            const uint64_t slot = op < a.nslots ? op : op % a.nslots;
            dst[u] = (V *)(dbase + slot * dslot) + j;
            v[u] = __builtin_nontemporal_load((const V *)(sbase + slot * sslot) + j);
        }
        t += (uint64_t)U * team_waves;
    };
    auto store = [&](const V (&v)[U], V *const (&dst)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) __builtin_nontemporal_store(v[u], dst[u]);
    };
    if (sets) {
        V va[U], vb[U];
        V *da[U], *db[U];
        load(va, da);
        for (;;) {
            if (sets == 1) { store(va, da); break; }
            load(vb, db);
            store(va, da);
            if (sets == 2) { store(vb, db); break; }
            load(va, da);
            store(vb, db);
            sets -= 2;
        }
    }
    for (uint32_t r = 0; r < rest; ++r, t += team_waves) {
        const uint64_t op_ = t * per_wave + sub;
        const uint64_t op = op_ < last_op ? op_ : last_op;
        const uint64_t slot = op < a.nslots ? op : op % a.nslots;
        __builtin_nontemporal_store(__builtin_nontemporal_load((const V *)(sbase + slot * sslot) + j), (V *)(dbase + slot * dslot) + j);
    }
}

__global__ __launch_bounds__(256) void k_copy_sweep(Ctx c, SweepArgs a)
{
    const uint32_t pe = blockIdx.x / a.wgs_per_pe;
    const uint32_t wg = blockIdx.x % a.wgs_per_pe;
    const uint32_t peer = (pe + 1) % (uint32_t)c.npes;
    const uint32_t lane = threadIdx.x & 63, waves_per_wg = blockDim.x >> 6;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint64_t team_waves = (uint64_t)a.wgs_per_pe * waves_per_wg;
    const uint64_t my_wave = (uint64_t)wg * waves_per_wg + wave;
    const bool contiguous = a.kind <= SHMEM_OP_GET;
    const uint64_t per_chunk = contiguous ? CHUNK_BYTES : CHUNK_ELEMS;
    const uint64_t chunks = (a.count + per_chunk - 1) / per_chunk;
    const uint64_t tasks = chunks * a.ops_per_pe;
    uint8_t *const lbase = ptr(c, a.local_off, pe);
    uint8_t *const rbase = ptr(c, a.remote_off, peer);
    // a message that one wave instruction covers (64 lanes x 16 bytes, or x 8 where only that alignment holds)
    const uint64_t align_bits = a.count | a.local_slot | a.remote_slot | a.local_off | a.remote_off;
    if (contiguous && (align_bits & 15) == 0 && a.count <= 2 * SMALL_MSG) {
        sweep_small<u32x4>(a, lbase, rbase, my_wave, team_waves, lane);
        return;
    }
    if (contiguous && (align_bits & 7) == 0 && a.count <= SMALL_MSG) {
        sweep_small<u32x2>(a, lbase, rbase, my_wave, team_waves, lane);
        return;
    }
    if (contiguous && a.count > 2 * SMALL_MSG && (align_bits & 15) == 0) {
        if (a.count > 4096 && a.count % 4096) {
            sweep_pipelined_ragged(a, lbase, rbase, my_wave, team_waves, lane);
            return;
        }
        // whole multiples of 4 KiB, and messages under 4 KiB: the leading multiple of 1 KiB goes through
        // the pipelined loop, as 4 KiB wave tasks (the fastest size) or as one task of 2 KiB and / or one
        // of 1 KiB per message ...
        const uint64_t body = a.count & ~1023ull, tail_vecs = (a.count - body) / 16;
        const uint64_t body4 = body & ~4095ull;
        if (body4) sweep_pipelined<4>(a, 0, body4, lbase, rbase, my_wave, team_waves, lane);
        if (body & 2048) sweep_pipelined<2>(a, body4, 2048, lbase, rbase, my_wave, team_waves, lane);
        if (body & 1024) sweep_pipelined<1>(a, body4 + (body & 2048), 1024, lbase, rbase, my_wave, team_waves, lane);
        // ... and what is left of each (under 1 KiB, e.g. the 16 metadata bytes of a 14,352-byte MoE
        // message) with one vector per lane
        if (tail_vecs) {
            for (uint64_t op = my_wave; op < a.ops_per_pe; op += team_waves) {
                const uint64_t slot = op % a.nslots;
                u32x4 *l = (u32x4 *)(lbase + slot * a.local_slot + body) + lane;
                u32x4 *r = (u32x4 *)(rbase + slot * a.remote_slot + body) + lane;
                if (lane < tail_vecs) {
                    if (a.kind == SHMEM_OP_PUT) __builtin_nontemporal_store(__builtin_nontemporal_load(l), r);
                    else __builtin_nontemporal_store(__builtin_nontemporal_load(r), l);
                }
            }
        }
        return;
    }
    for (uint64_t t = my_wave; t < tasks; t += team_waves) {
        const uint64_t op = t / chunks, ch = t - op * chunks;
        const uint64_t slot = op % a.nslots;
        uint8_t *l = lbase + slot * a.local_slot;
        uint8_t *r = rbase + slot * a.remote_slot;
        const uint64_t first = ch * per_chunk;
        const uint64_t cnt = a.count - first < per_chunk ? a.count - first : per_chunk;
        if (contiguous) {
            if (a.kind == SHMEM_OP_PUT) copy(r + first, l + first, cnt, lane, 64);
            else copy(l + first, r + first, cnt, lane, 64);
        } else {
            const uint64_t eb = a.elem_bytes;
            uint8_t *lp = l + first * (uint64_t)a.local_stride * eb;
            uint8_t *rp = r + first * (uint64_t)a.remote_stride * eb;
            if (a.kind == SHMEM_OP_IPUT) strided(rp, lp, a.remote_stride, a.local_stride, cnt, a.elem_bytes, lane, 64);
            else strided(lp, rp, a.local_stride, a.remote_stride, cnt, a.elem_bytes, lane, 64);
        }
    }
}

}  // namespace shmemx

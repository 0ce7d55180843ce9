// Atomic-memory-operation kernels: a stand-alone AMO and the batched forms
// (direct, and with workgroup-level combining in LDS).
#pragma once
#include "../../include/mi_shmem.h"
#include "../../include/mi_shmemx.hpp"

namespace shmemx {

struct AmoArgs {
    int kind;
    uint64_t ctr_off;            // symmetric offset of the counter array
    uint64_t T;                  // counters per PE
    const int32_t *pe;           // target PE of op i
    const uint32_t *idx;         // counter index of op i
    const uint64_t *a, *b;       // operands
    uint64_t *old;               // fetched values (may be null)
    uint64_t n, per_pe;          // ops in total / ops issued per PE (block layout)
    uint32_t wgs_per_pe;
};

// store `val` if the word is 0 or larger, through a compare-swap retry loop
__device__ __forceinline__ uint64_t min_cas_loop(uint64_t *w, uint64_t val)
{
    uint64_t cur = atomic_fetch(w);
    while (cur == 0 || cur > val) {
        const uint64_t seen = atomic_compare_swap(w, cur, val);
        if (seen == cur) break;
        cur = seen;
    }
    return cur;
}

__device__ __forceinline__ uint64_t amo_apply(int kind, uint64_t *w, uint64_t a, uint64_t b)
{
    switch (kind) {
    case SHMEM_AMO_FETCH_ADD: return atomic_fetch_add(w, a);
    case SHMEM_AMO_COMPARE_SWAP: return atomic_compare_swap(w, a, b);
    case SHMEM_AMO_FETCH_OR: return atomic_fetch_or(w, a);
    default: return min_cas_loop(w, a);
    }
}

__global__ void k_amo_single(int kind, uint64_t *target, uint64_t a, uint64_t b, uint64_t *result)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const uint64_t seen = amo_apply(kind, target, a, b);
        if (result) *result = seen;
    }
}

// One hardware atomic per op.  PE team p issues ops [p * per_pe, (p+1) * per_pe);
// consecutive lanes take consecutive ops, so the operand streams are coalesced.
__global__ __launch_bounds__(256) void k_amo_batch(Ctx c, AmoArgs g)
{
    const uint32_t pe_self = blockIdx.x / g.wgs_per_pe, wg = blockIdx.x % g.wgs_per_pe;
    const uint64_t begin = (uint64_t)pe_self * g.per_pe;
    const uint64_t end = begin + g.per_pe < g.n ? begin + g.per_pe : g.n;
    for (uint64_t i = begin + (uint64_t)wg * blockDim.x + threadIdx.x; i < end; i += (uint64_t)g.wgs_per_pe * blockDim.x) {
        const uint32_t tp = (uint32_t)g.pe[i], ix = g.idx[i];
        if (tp >= (uint32_t)c.npes || ix >= g.T) { report(c, DEV_ERR_BAD_TARGET, i); continue; }
        uint64_t *w = (uint64_t *)ptr(c, g.ctr_off + 8ull * ix, tp);
        const uint64_t seen = amo_apply(g.kind, w, g.a[i], g.kind == SHMEM_AMO_COMPARE_SWAP ? g.b[i] : 0);
        if (g.old) g.old[i] = seen;
    }
}

// Workgroup-level combining.  A pass takes AGG_OPS ops of the workgroup.  Each
// op finds (or claims) the LDS slot of its target word in a small open-addressed
// table keyed by pe * T + idx and applies its operand there with a returning
// LDS atomic, which hands it its position inside the group.  The lane that
// claimed the slot then issues ONE hardware atomic with the group's combined
// operand; every op derives its fetched value from the returned base and its
// position.  The group's ops thus behave as if they ran back to back.
constexpr uint32_t AGG_PER_THREAD = 4;
constexpr uint32_t AGG_SLOTS = 2048;        // >= 2 * 256 * AGG_PER_THREAD
constexpr uint32_t AGG_EMPTY = 0xFFFFFFFFu;

__global__ __launch_bounds__(256) void k_amo_batch_agg(Ctx c, AmoArgs g)
{
    __shared__ uint32_t s_key[AGG_SLOTS];
    __shared__ unsigned long long s_val[AGG_SLOTS];
    __shared__ unsigned long long s_base[AGG_SLOTS];
    const uint32_t pe_self = blockIdx.x / g.wgs_per_pe, wg = blockIdx.x % g.wgs_per_pe;
    const uint64_t begin = (uint64_t)pe_self * g.per_pe;
    const uint64_t end = begin + g.per_pe < g.n ? begin + g.per_pe : g.n;
    const uint64_t pass_ops = (uint64_t)blockDim.x * AGG_PER_THREAD;
    const unsigned long long ident = g.kind == SHMEM_AMO_MIN_CAS_LOOP ? ~0ull : 0ull;
    for (uint64_t p0 = begin + (uint64_t)wg * pass_ops; p0 < end; p0 += (uint64_t)g.wgs_per_pe * pass_ops) {
        for (uint32_t s = threadIdx.x; s < AGG_SLOTS; s += blockDim.x) { s_key[s] = AGG_EMPTY; s_val[s] = ident; }
        __syncthreads();
        uint32_t slot[AGG_PER_THREAD];
        bool owner[AGG_PER_THREAD];
        unsigned long long pos[AGG_PER_THREAD];
        uint64_t *word[AGG_PER_THREAD];
#pragma unroll
        for (uint32_t j = 0; j < AGG_PER_THREAD; ++j) {
            const uint64_t i = p0 + (uint64_t)j * blockDim.x + threadIdx.x;
            slot[j] = AGG_EMPTY; owner[j] = false; pos[j] = 0; word[j] = nullptr;
            if (i >= end) continue;
            const uint32_t tp = (uint32_t)g.pe[i], ix = g.idx[i];
            if (tp >= (uint32_t)c.npes || ix >= g.T) { report(c, DEV_ERR_BAD_TARGET, i); continue; }
            const uint32_t key = tp * (uint32_t)g.T + ix;
            word[j] = (uint64_t *)ptr(c, g.ctr_off + 8ull * ix, tp);
            uint32_t h = (key * 0x9E3779B1u) >> 21;            // 11 bits -> [0, AGG_SLOTS)
            for (;;) {
                const uint32_t prev = atomicCAS(&s_key[h], AGG_EMPTY, key);
                if (prev == AGG_EMPTY) { owner[j] = true; break; }
                if (prev == key) break;
                h = (h + 1) & (AGG_SLOTS - 1);
            }
            slot[j] = h;
            const unsigned long long a = g.a[i];
            if (g.kind == SHMEM_AMO_FETCH_ADD) pos[j] = atomicAdd(&s_val[h], a);
            else if (g.kind == SHMEM_AMO_FETCH_OR) pos[j] = atomicOr(&s_val[h], a);
            else pos[j] = atomicMin(&s_val[h], a);
        }
        __syncthreads();
#pragma unroll
        for (uint32_t j = 0; j < AGG_PER_THREAD; ++j)
            if (owner[j]) s_base[slot[j]] = amo_apply(g.kind, word[j], s_val[slot[j]], 0);
        __syncthreads();
#pragma unroll
        for (uint32_t j = 0; j < AGG_PER_THREAD; ++j) {
            const uint64_t i = p0 + (uint64_t)j * blockDim.x + threadIdx.x;
            if (slot[j] == AGG_EMPTY || !g.old) continue;
            const unsigned long long base = s_base[slot[j]];
            // what the word held just before this op, the group's ops taken in the order in which they reached
            // the LDS slot: the base plus / or-ed with / lowered by what the earlier ones brought (pos is the
            // slot's value before this op; for the minimum it starts at all ones = nothing yet, and a word of 0
            // counts as empty)
            unsigned long long seen;
            if (g.kind == SHMEM_AMO_FETCH_ADD) seen = base + pos[j];
            else if (g.kind == SHMEM_AMO_FETCH_OR) seen = base | pos[j];
            else seen = pos[j] == ~0ull ? base : (base == 0 || pos[j] < base ? pos[j] : base);
            g.old[i] = seen;
        }
        __syncthreads();
    }
}

}  // namespace shmemx

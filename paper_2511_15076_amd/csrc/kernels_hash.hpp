// Distributed open-addressing hash table: insert by compare-swap, lookup by get.
#pragma once
#include "../../include/mi_shmem.h"
#include "../../include/mi_shmemx.hpp"

namespace shmemx {

struct HashArgs {
    uint64_t table_off;          // symmetric offset of the table
    uint32_t slots;              // slots per PE
    const uint64_t *keys;
    uint64_t n, per_pe;          // keys in total / keys held per PE (block layout)
    uint8_t *out;                // status (insert) or found flag (lookup)
    uint32_t wgs_per_pe;
};

// SplitMix64 finaliser
__device__ __forceinline__ uint64_t hash_mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// owner = h mod npes, home = (h / npes) mod slots; shifts and masks when the
// divisors are powers of two (they are in the benchmark shapes)
__device__ __forceinline__ void hash_place(const Ctx &c, uint32_t slots, uint64_t key, uint32_t *owner, uint32_t *home)
{
    const uint64_t h = hash_mix64(key);
    const uint32_t np = (uint32_t)c.npes;
    uint64_t q;
    if ((np & (np - 1)) == 0) { *owner = (uint32_t)h & (np - 1); q = h >> __builtin_ctz(np); }
    else { *owner = (uint32_t)(h % np); q = h / np; }
    *home = (slots & (slots - 1)) == 0 ? (uint32_t)q & (slots - 1) : (uint32_t)(q % slots);
}

// Keys in flight per lane: the first probe of each is issued before any of them
// is examined, so a lane keeps HASH_KIF independent random line fetches going.
constexpr int HASH_KIF = 4;

__global__ __launch_bounds__(256) void k_hash_insert(Ctx c, HashArgs g)
{
    const uint32_t pe_self = blockIdx.x / g.wgs_per_pe, wg = blockIdx.x % g.wgs_per_pe;
    const uint64_t begin = (uint64_t)pe_self * g.per_pe;
    const uint64_t end = begin + g.per_pe < g.n ? begin + g.per_pe : g.n;
    const uint64_t stride = (uint64_t)g.wgs_per_pe * blockDim.x;
    for (uint64_t i0 = begin + (uint64_t)wg * blockDim.x + threadIdx.x; i0 < end; i0 += stride * HASH_KIF) {
        uint64_t key[HASH_KIF], seen[HASH_KIF], *table[HASH_KIF];
        uint32_t slot[HASH_KIF];
        bool live[HASH_KIF];
#pragma unroll
        for (int k = 0; k < HASH_KIF; ++k) {
            const uint64_t i = i0 + k * stride;
            live[k] = i < end;
            key[k] = live[k] ? __builtin_nontemporal_load(g.keys + i) : 1;
        }
#pragma unroll
        for (int k = 0; k < HASH_KIF; ++k) {
            uint32_t owner;
            hash_place(c, g.slots, key[k], &owner, &slot[k]);
            table[k] = (uint64_t *)ptr(c, g.table_off, owner);
            seen[k] = 1;
            if (live[k] && key[k] != 0) seen[k] = table[k][slot[k]];      // first probe
        }
#pragma unroll
        for (int k = 0; k < HASH_KIF; ++k) {
            if (!live[k]) continue;
            const uint64_t i = i0 + k * stride;
            if (key[k] == 0) { report(c, DEV_ERR_BAD_OP, i); continue; }
            uint8_t st = SHMEM_HASH_FULL;
            uint64_t cur = seen[k];
            uint32_t sl = slot[k];
            for (uint32_t j = 0; j < g.slots; ++j) {
                // A non-zero word never changes again, so a plain read that shows one is
                // final; only an empty-looking slot needs the compare-swap.
                if (j) cur = table[k][sl];
                if (cur == 0) cur = atomic_compare_swap(&table[k][sl], 0, key[k]);
                if (cur == 0) { st = SHMEM_HASH_INSERTED; break; }
                if (cur == key[k]) { st = SHMEM_HASH_DUPLICATE; break; }
                sl = sl + 1 == g.slots ? 0 : sl + 1;
            }
            if (g.out) g.out[i] = st;
        }
    }
}

__global__ __launch_bounds__(256) void k_hash_lookup(Ctx c, HashArgs g)
{
    const uint32_t pe_self = blockIdx.x / g.wgs_per_pe, wg = blockIdx.x % g.wgs_per_pe;
    const uint64_t begin = (uint64_t)pe_self * g.per_pe;
    const uint64_t end = begin + g.per_pe < g.n ? begin + g.per_pe : g.n;
    const uint64_t stride = (uint64_t)g.wgs_per_pe * blockDim.x;
    for (uint64_t i0 = begin + (uint64_t)wg * blockDim.x + threadIdx.x; i0 < end; i0 += stride * HASH_KIF) {
        uint64_t key[HASH_KIF], seen[HASH_KIF];
        const uint64_t *table[HASH_KIF];
        uint32_t slot[HASH_KIF];
        bool live[HASH_KIF];
#pragma unroll
        for (int k = 0; k < HASH_KIF; ++k) {
            const uint64_t i = i0 + k * stride;
            live[k] = i < end;
            key[k] = live[k] ? __builtin_nontemporal_load(g.keys + i) : 0;
        }
#pragma unroll
        for (int k = 0; k < HASH_KIF; ++k) {
            uint32_t owner;
            hash_place(c, g.slots, key[k], &owner, &slot[k]);
            table[k] = (const uint64_t *)ptr(c, g.table_off, owner);
            seen[k] = 0;
            if (live[k]) seen[k] = table[k][slot[k]];                     // an 8-byte get from the owner
        }
#pragma unroll
        for (int k = 0; k < HASH_KIF; ++k) {
            if (!live[k]) continue;
            uint8_t found = 0;
            uint64_t cur = seen[k];
            uint32_t sl = slot[k];
            for (uint32_t j = 0; j < g.slots; ++j) {
                if (j) cur = table[k][sl];
                if (cur == key[k]) { found = 1; break; }
                if (cur == 0) break;
                sl = sl + 1 == g.slots ? 0 : sl + 1;
            }
            g.out[i0 + k * stride] = found;
        }
    }
}

// Lookup for tables whose slot count per PE is a multiple of 8: a probe sequence is read a whole
// 64-byte sector (8 slots) at a time, the sector that holds the current slot.  The table is far larger
// than the caches and tens of thousands of probe sequences are in flight per die, so a second 8-byte
// probe a moment later finds its sector evicted and fetches it from memory again (measured: two sector
// fetches per key at load 0.5, and a lookup rate that falls with the mean chain length).  One 64-byte
// read brings everything a sector can contribute; the walk goes on in the next sector only when the
// chain runs off the end (the table keeps plain linear probing: what is found is unchanged).  Read by
// one lane as four 16-byte loads this was slower than the 8-byte probes (41 against 50 G lookups/s on
// single-probe chains): four instructions and four cache look-ups per key.
constexpr int HASH_SECTOR = 8;   // slots per 64-byte sector

// Four neighbouring lanes (a quad) look one key up: each reads 16 bytes of the sector, so a wave
// instruction requests 16 whole sectors, one coalesced 64-byte access per key.  Every lane classifies
// its two slots (2 bits each: 1 = the key, 2 = empty, 0 = another key or before the start), the quad
// ORs the codes with two DPP quad permutes and the lowest non-zero field decides.
__device__ __forceinline__ uint32_t quad_or(uint32_t v)
{
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, false);   // lanes ^ 1
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, false);   // lanes ^ 2
    return v;
}

template <int KIF>
__global__ __launch_bounds__(256) void k_hash_lookup_sectors(Ctx c, HashArgs g)
{
    const uint32_t pe_self = blockIdx.x / g.wgs_per_pe, wg = blockIdx.x % g.wgs_per_pe;
    const uint64_t begin = (uint64_t)pe_self * g.per_pe;
    const uint64_t end = begin + g.per_pe < g.n ? begin + g.per_pe : g.n;
    const uint32_t q4 = threadIdx.x & 3, quads = blockDim.x >> 2;
    const uint64_t stride = (uint64_t)g.wgs_per_pe * quads;
    for (uint64_t i0 = begin + (uint64_t)wg * quads + (threadIdx.x >> 2); i0 < end; i0 += stride * KIF) {
        uint64_t key[KIF];
        const u32x4 *table[KIF];           // the owner's table as 16-byte vectors, offset to this lane's quarter
        uint32_t slot[KIF];
        u32x4 w[KIF];
        bool live[KIF];
#pragma unroll
        for (int k = 0; k < KIF; ++k) {
            const uint64_t i = i0 + k * stride;
            live[k] = i < end;
            key[k] = live[k] ? __builtin_nontemporal_load(g.keys + i) : 0;
        }
#pragma unroll
        for (int k = 0; k < KIF; ++k) {
            uint32_t owner;
            hash_place(c, g.slots, key[k], &owner, &slot[k]);
            table[k] = (const u32x4 *)ptr(c, g.table_off, owner) + q4;
            w[k] = live[k] ? table[k][(size_t)(slot[k] / HASH_SECTOR) * 4] : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int k = 0; k < KIF; ++k) {
            if (!live[k]) continue;                           // the same for all four lanes of a quad
            const uint32_t klo = (uint32_t)key[k], khi = (uint32_t)(key[k] >> 32);
            uint32_t sector = slot[k] / HASH_SECTOR, start = slot[k] % HASH_SECTOR;
            uint32_t found = 0;
            for (uint32_t probed = 0; probed < g.slots;) {
                uint32_t code = 0;
                if (2 * q4 >= start) code |= ((w[k].x == klo && w[k].y == khi) ? 1u : (w[k].x | w[k].y) == 0 ? 2u : 0u) << (4 * q4);
                if (2 * q4 + 1 >= start) code |= ((w[k].z == klo && w[k].w == khi) ? 1u : (w[k].z | w[k].w) == 0 ? 2u : 0u) << (4 * q4 + 2);
                code = quad_or(code);
                if (code) { found = (code >> (__builtin_ctz(code) & ~1)) & 1; break; }
                probed += HASH_SECTOR - start;
                start = 0;
                sector = sector + 1 == g.slots / HASH_SECTOR ? 0 : sector + 1;
                w[k] = table[k][(size_t)sector * 4];
            }
            if (q4 == 0) g.out[i0 + k * stride] = (uint8_t)found;
        }
    }
}

}  // namespace shmemx

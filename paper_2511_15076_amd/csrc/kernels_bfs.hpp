// Level-synchronous BFS over a 1D block vertex partition, built on the
// one-sided primitives: fetch_or claims a vertex in its owner's bitmap,
// fetch_add reserves a slot in the owner's next-frontier queue, puts deliver
// the vertex, its parent and its level.  One launch per level; the kernel
// boundary is the quiet + barrier_all between levels.
#pragma once
#include "../../include/mi_shmem.h"
#include "shmemx.hpp"

namespace shmemx {

struct BfsState {
    uint32_t nverts, vpp;        // vertices in total / per PE (block partition)
    uint64_t words;              // bitmap words per PE
    int shift;                   // log2(vpp) if vpp is a power of two, else -1
    const uint64_t *row_off;     // CSR row offsets (PE p reads rows of its own vertices)
    const uint32_t *nbr;         // CSR neighbours
    // symmetric offsets of the per-PE state
    uint64_t bitmap_off, level_off, parent_off, queue_off[2], hub_off, tails_off;
    uint64_t filter_off;         // NXCD private copies of the bitmap (initiator-side cache, see bfs_visit)
    uint32_t wgs_per_pe;
};

// words inside the per-PE tails block (uint64 each)
enum : uint32_t { T_TAIL0 = 0 /* three rotating frontier counts */, T_HUBS = 4 };

constexpr uint32_t HUB_DEGREE = 2048;  // rows at least this long are expanded by the whole team
constexpr uint32_t NXCD = 8;           // accelerator dies, each with a private L2

// Index of the die this wave runs on (XCC_ID hardware register, 4 bits).
__device__ __forceinline__ uint32_t xcd_id() { return __builtin_amdgcn_s_getreg(20 | (0 << 6) | ((4 - 1) << 11)) & (NXCD - 1); }

__device__ __forceinline__ uint32_t bfs_owner(const BfsState &s, uint32_t v)
{
    return s.shift >= 0 ? v >> s.shift : v / s.vpp;
}
__device__ __forceinline__ uint64_t *bfs_tails(const Ctx &c, const BfsState &s, uint32_t pe)
{
    return (uint64_t *)ptr(c, s.tails_off, pe);
}

// Every owner clears its slice; the root's owner seeds the search.
__global__ __launch_bounds__(256) void k_bfs_init(Ctx c, BfsState s, uint32_t root)
{
    const uint32_t pe = blockIdx.x / s.wgs_per_pe, wg = blockIdx.x % s.wgs_per_pe;
    const uint64_t rank = (uint64_t)wg * blockDim.x + threadIdx.x, size = (uint64_t)s.wgs_per_pe * blockDim.x;
    const uint32_t ro = bfs_owner(s, root), rl = root - ro * s.vpp;
    uint64_t *bm = (uint64_t *)ptr(c, s.bitmap_off, pe);
    int32_t *lv = (int32_t *)ptr(c, s.level_off, pe);
    uint32_t *pr = (uint32_t *)ptr(c, s.parent_off, pe);
    for (uint64_t w = rank; w < s.words; w += size)
        bm[w] = (pe == ro && w == (rl >> 6)) ? 1ull << (rl & 63) : 0ull;
    uint64_t *flt = (uint64_t *)ptr(c, s.filter_off, pe);
    for (uint64_t w = rank; w < s.words * NXCD; w += size) flt[w] = 0;
    for (uint64_t l = rank; l < s.vpp; l += size) {
        const bool is_root = pe == ro && l == rl;
        lv[l] = is_root ? 0 : -1;
        pr[l] = is_root ? root : SHMEM_BFS_NONE;
    }
    if (rank == 0) {
        uint64_t *t = bfs_tails(c, s, pe);
        t[T_TAIL0 + 0] = pe == ro ? 1 : 0; t[T_TAIL0 + 1] = 0; t[T_TAIL0 + 2] = 0; t[T_HUBS] = 0;
        if (pe == ro) ((uint32_t *)ptr(c, s.queue_off[0], pe))[0] = root;
        if (pe == 0) c.scratch[W_WORK + 1] = 0;  // degree sum of reached vertices
    }
}

// Visit neighbour v of frontier vertex u (lanes with active == false only take
// part in the wave-wide steps).
//
// Test before set: the fetch_or on the owner's bitmap is the claim, but most
// probes find a vertex that is already claimed.  Atomics resolve beyond the
// per-die L2s, and a plain read of the bitmap word may hit a line that this
// die's L2 fetched before the bit was set, so a plain test of the bitmap itself
// stays blind to everything claimed during the current level.  Each die
// therefore keeps a private copy of the bitmap that only its own waves read and
// write with plain accesses (coherent inside one L2): a bit is set there after
// a fetch_or has shown the vertex to be claimed, so a set bit is always true
// and a missing bit (first probe from this die, or a lost racy update) only
// costs one more fetch_or.
__device__ __forceinline__ void bfs_visit(const Ctx &c, const BfsState &s, uint32_t xcd, bool active, uint32_t v,
                                          uint32_t u, uint32_t L)
{
    bool won = false;
    uint32_t o = 0, l = 0;
    if (active) {
        o = bfs_owner(s, v);
        l = v - o * s.vpp;
        const uint64_t bit = 1ull << (l & 63);
        uint64_t *f = (uint64_t *)ptr(c, s.filter_off, o) + (uint64_t)xcd * s.words + (l >> 6);
        const uint64_t known = *f;
        if (!(known & bit)) {
            uint64_t *w = (uint64_t *)ptr(c, s.bitmap_off, o) + (l >> 6);
            const uint64_t old = atomic_fetch_or(w, bit);
            won = !(old & bit);
            *f = known | old | bit;      // everything the fetch_or showed to be claimed
        }
    }
    // winners that share an owner reserve their queue slots with one fetch_add
    uint64_t m = ballot(won);
    const uint32_t lane = lane_id();
    while (m) {
        const uint32_t leader = (uint32_t)__builtin_ctzll(m);
        const uint32_t ol = bcast32(o, leader);
        const uint64_t grp = ballot(won && o == ol);
        uint64_t base = 0;
        if (lane == leader)
            base = atomic_fetch_add(bfs_tails(c, s, ol) + T_TAIL0 + (L + 1) % 3, (uint64_t)__builtin_popcountll(grp));
        base = bcast64(base, leader);
        if (won && o == ol) {
            const uint64_t slot = base + rank_in(grp);
            ((uint32_t *)ptr(c, s.queue_off[(L + 1) & 1], ol))[slot] = v;   // put v
            ((uint32_t *)ptr(c, s.parent_off, ol))[l] = u;                  // put parent
            ((int32_t *)ptr(c, s.level_off, ol))[l] = (int32_t)(L + 1);     // put level
        }
        m &= ~grp;
    }
}

// Expand level L.  A wave takes 64 frontier vertices at a time (coalesced queue
// read, 64 row lookups in flight), then walks their rows one after the other
// with all lanes; very long rows are set aside for k_bfs_hubs.
__global__ __launch_bounds__(256) void k_bfs_expand(Ctx c, BfsState s, uint32_t L)
{
    const uint32_t pe = blockIdx.x / s.wgs_per_pe, wg = blockIdx.x % s.wgs_per_pe;
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wpw = blockDim.x >> 6;
    const uint64_t team_waves = (uint64_t)s.wgs_per_pe * wpw, my_wave = (uint64_t)wg * wpw + wave;
    const uint32_t xcd = xcd_id();
    uint64_t *tails = bfs_tails(c, s, pe);
    const uint64_t cnt = tails[T_TAIL0 + L % 3];
    const uint32_t *queue = (const uint32_t *)ptr(c, s.queue_off[L & 1], pe);
    uint32_t *hubs = (uint32_t *)ptr(c, s.hub_off, pe);
    uint64_t degsum = 0;
    for (uint64_t base = my_wave * 64; base < cnt; base += team_waves * 64) {
        const bool valid = base + lane < cnt;
        uint32_t u = 0, deg = 0;
        uint64_t r0 = 0;
        if (valid) {
            u = queue[base + lane];
            r0 = s.row_off[u];
            deg = (uint32_t)(s.row_off[u + 1] - r0);
        }
        degsum += deg;
        const bool hub = deg >= HUB_DEGREE;
        const uint64_t hm = ballot(hub);
        if (hm) {
            const uint32_t leader = (uint32_t)__builtin_ctzll(hm);
            uint64_t hb = 0;
            if (lane == leader) hb = atomic_fetch_add(tails + T_HUBS, (uint64_t)__builtin_popcountll(hm));
            hb = bcast64(hb, leader);
            if (hub) hubs[hb + rank_in(hm)] = u;
        }
        uint64_t todo = ballot(valid && !hub && deg > 0);
        while (todo) {
            const uint32_t j = (uint32_t)__builtin_ctzll(todo);
            todo &= todo - 1;
            const uint32_t uj = bcast32(u, j), dj = bcast32(deg, j);
            const uint64_t rj = bcast64(r0, j);
            for (uint32_t t0 = 0; t0 < dj; t0 += 64) {
                const bool act = t0 + lane < dj;
                const uint32_t v = act ? s.nbr[rj + t0 + lane] : 0;
                bfs_visit(c, s, xcd, act, v, uj, L);
            }
        }
    }
    // degree sum of this level's frontier -> traversed-edge count
    for (int off = 32; off > 0; off >>= 1) degsum += __shfl_down(degsum, off, 64);
    if (lane == 0 && degsum) atomic_fetch_add(&c.scratch[W_WORK + 1], degsum);
}

// Long rows of level L: all waves of the owner's team stride over each of them.
__global__ __launch_bounds__(256) void k_bfs_hubs(Ctx c, BfsState s, uint32_t L)
{
    const uint32_t pe = blockIdx.x / s.wgs_per_pe, wg = blockIdx.x % s.wgs_per_pe;
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wpw = blockDim.x >> 6;
    const uint64_t team_waves = (uint64_t)s.wgs_per_pe * wpw, my_wave = (uint64_t)wg * wpw + wave;
    const uint32_t xcd = xcd_id();
    const uint64_t nh = bfs_tails(c, s, pe)[T_HUBS];
    const uint32_t *hubs = (const uint32_t *)ptr(c, s.hub_off, pe);
    for (uint64_t h = 0; h < nh; ++h) {
        const uint32_t u = hubs[h];
        const uint64_t r0 = s.row_off[u], deg = s.row_off[u + 1] - r0;
        for (uint64_t t0 = my_wave * 64; t0 < deg; t0 += team_waves * 64) {
            const bool act = t0 + lane < deg;
            const uint32_t v = act ? s.nbr[r0 + t0 + lane] : 0;
            bfs_visit(c, s, xcd, act, v, u, L);
        }
    }
}

// Level epilogue (one wave): total size of frontier `next`, reset of the hub
// lists and of the count that level next+1 will fill.
__global__ void k_bfs_count(Ctx c, BfsState s, uint32_t next)
{
    uint64_t total = 0;
    for (uint32_t pe = threadIdx.x; pe < (uint32_t)c.npes; pe += blockDim.x) {
        uint64_t *t = bfs_tails(c, s, pe);
        total += t[T_TAIL0 + next % 3];
        t[T_TAIL0 + (next + 1) % 3] = 0;
        t[T_HUBS] = 0;
    }
    for (int off = 32; off > 0; off >>= 1) total += __shfl_down(total, off, 64);
    if (threadIdx.x == 0) c.scratch[W_WORK] = total;
}

// Every owner copies its level / parent slice into the caller's flat arrays.
__global__ __launch_bounds__(256) void k_bfs_gather(Ctx c, BfsState s, int32_t *level, uint32_t *parent)
{
    const uint32_t pe = blockIdx.x / s.wgs_per_pe, wg = blockIdx.x % s.wgs_per_pe;
    const uint64_t rank = (uint64_t)wg * blockDim.x + threadIdx.x, size = (uint64_t)s.wgs_per_pe * blockDim.x;
    const uint64_t first = (uint64_t)pe * s.vpp;
    if (first >= s.nverts) return;
    const uint64_t cnt = s.nverts - first < s.vpp ? s.nverts - first : s.vpp;
    if (level) copy((uint8_t *)(level + first), ptr(c, s.level_off, pe), cnt * 4, rank, size);
    if (parent) copy((uint8_t *)(parent + first), ptr(c, s.parent_off, pe), cnt * 4, rank, size);
}

}  // namespace shmemx

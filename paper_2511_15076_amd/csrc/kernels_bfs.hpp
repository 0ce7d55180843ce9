// Level-synchronous BFS over a 1D block vertex partition, built on the
// one-sided primitives: fetch_or claims a vertex in its owner's bitmap,
// fetch_add reserves slots in the owner's next-frontier queue, puts deliver
// the vertex, its parent and its level.  One set of launches per level; the
// kernel boundary is the quiet + barrier_all between levels.
//
// Work distribution inside a PE team:
//   k_bfs_expand   a wave takes 64 frontier vertices, sets long rows aside and
//                  expands the short ones packed: a wave-wide prefix sum over
//                  the row lengths lets every lane take edges, whatever the
//                  length mix (R-MAT degrees are heavily skewed);
//   k_bfs_bigscan  prefix sum over the long rows' segment counts (one
//                  workgroup per PE);
//   k_bfs_big      the team's waves split the long rows' 512-edge segments
//                  evenly (each wave takes a run of consecutive segments);
//   k_bfs_level_end  frontier bitmap / degree sum (direction-optimising modes); its last workgroup
//                  totals the next frontier, resets counters and hands the counts to the host.
#pragma once
#include "../../include/mi_shmem.h"
#include "../../include/mi_shmemx.hpp"

namespace shmemx {

struct BfsState {
    uint32_t nverts, vpp;        // vertices in total / per PE (block partition)
    uint64_t words;              // bitmap words per PE
    int shift;                   // log2(vpp) if vpp is a power of two, else -1
    // The search runs on the library's own numbering of the vertices (see k_bfs_relabel): nverts counts its
    // vertices (npes * vpp: every PE a full block), row_off / nbr are the graph in that numbering, to_orig[i] is the
    // caller's number of vertex i (SHMEM_BFS_NONE for the padding at the end of a block, which has no edges).
    const uint64_t *row_off;     // CSR row offsets (PE p reads rows of its own vertices)
    const uint32_t *nbr;         // CSR neighbours
    const uint32_t *to_orig;
    // symmetric offsets of the per-PE state
    uint64_t bitmap_off, pl_off, queue_off[2], big_off, bigscan_off, tails_off;   // pl: (parent, level) pairs, 8 bytes per vertex
    uint64_t filter_off;         // NXCD private copies of the bitmap (initiator-side cache, see bfs_probe)
    uint64_t front_off, prev_off; // frontier bitmap and the bitmap as of the previous level (bottom-up levels; prev in the claim bitmap's layout)
    uint64_t linked_off;          // bit set = the vertex has at least one neighbour (never changes)
    uint32_t wgs_per_pe;
    // Layout of the bitmap that takes the claims (bitmap_off only; the die copies, front, prev and linked keep
    // word w at place w): 0 = word w at place w, else log2 of the block of words inside which 16 consecutive words
    // are spread over 16 different 128-byte lines (see bfs_vis_word).
    uint32_t vis_block_log2;
};

// Place of bitmap word w (bits of local vertices 64 w .. 64 w + 63) in the owner's claim bitmap.  Atomics on ONE
// 128-byte line are served one after the other whatever words of the line they name (measured: 256 words take 3 G
// fetch_or/s when they fill 16 lines and 21 G/s on a line each), and in the degree-ranked numbering the
// best-connected vertices are the first words of every PE: side by side they would share a line per PE, which the
// claims of a level that expands a few hubs then queue up on.  Inside an aligned block of B words (B / 16 lines)
// word i of the block goes to line i mod (B / 16), slot i / (B / 16); a last, incomplete block stays as it is.
__device__ __forceinline__ uint64_t bfs_vis_word(const BfsState &s, uint64_t w)
{
    if (s.vis_block_log2 == 0) return w;
    const uint64_t B = 1ull << s.vis_block_log2, blk = w & ~(B - 1);
    if (blk + B > s.words) return w;
    const uint64_t i = w & (B - 1);
    return blk | ((i & ((B >> 4) - 1)) << 4) | (i >> (s.vis_block_log2 - 4));
}

// ... and back: the bitmap word that lives at place q
__device__ __forceinline__ uint64_t bfs_vis_word_at(const BfsState &s, uint64_t q)
{
    if (s.vis_block_log2 == 0) return q;
    const uint64_t B = 1ull << s.vis_block_log2, blk = q & ~(B - 1);
    if (blk + B > s.words) return q;
    return blk | ((q & 15) << (s.vis_block_log2 - 4)) | ((q & (B - 1)) >> 4);
}

// words inside the per-PE tails block (uint64 each)
enum : uint32_t { T_TAIL0 = 0 /* three rotating frontier counts */, T_NBIG = 4, T_NTASKS = 5,
                  T_ARRIVE = 6 /* workgroups of this PE that have finished the level-end kernel */,
                  // running degree sums, per PE and on a line of their own (adds on one address serialise at
                  // about 12 ns each: one word for the whole device cost 50 us per launch of 4096 waves)
                  T_DEG_EXPANDED = 16 /* frontiers expanded top-down */, T_DEG_FOUND = 17 /* frontiers discovered */,
                  T_FILL = 18 /* write position of k_bfs_fill_queue */,
                  // work handed out to the waves of the two top-down kernels of a level (reset with the level)
                  T_CLAIM_EXPAND = 24 /* batches of frontier vertices */, T_CLAIM_BIG = 25 /* runs of long-row segments */ };

constexpr uint32_t BIG_DEGREE = 512;   // rows at least this long go to k_bfs_big (128 to 512 measure alike, 1024 and 64 are 4 and 7 % slower)
// edges per lane in flight: four when short rows are expanded packed, eight in the long-row kernel (measured with
// 2 / 4 / 8 everywhere: the level that claims 7.5 M vertices 1.83 / 1.77 / 1.64 ms, the 7.5 M-vertex level of short rows
// 1.11 / 1.05 / 1.24)
constexpr uint32_t EPL_SHORT = 4, EPL_LONG = 8;
constexpr uint32_t SEG_EDGES = 64 * EPL_LONG;   // edges per long-row segment
constexpr uint32_t NXCD = 8;           // accelerator dies, each with a private L2
constexpr uint32_t STAGE_PES = 16;     // winners are staged in LDS when npes <= this
constexpr uint32_t STAGE_BLOCK = 64;   // staged vertices leave in blocks of this many (one 256-byte put)
constexpr uint32_t STAGE_CAP = STAGE_BLOCK + 64;   // per owner per wave: a partial block plus one entry per lane

// Index of the die this wave runs on (XCC_ID hardware register, 4 bits).
__device__ __forceinline__ uint32_t xcd_id()
{
    return __builtin_amdgcn_s_getreg(20 | (0 << 6) | ((4 - 1) << 11)) & (NXCD - 1);
}
__device__ __forceinline__ uint32_t bfs_owner(const BfsState &s, uint32_t v)
{
    return s.shift >= 0 ? v >> s.shift : v / s.vpp;
}
__device__ __forceinline__ uint64_t *bfs_tails(const Ctx &c, const BfsState &s, uint32_t pe)
{
    return (uint64_t *)ptr(c, s.tails_off, pe);
}

// Parent and level of a vertex are ONE 8-byte record in its owner's segment (parent in the low word, level in
// the high one): whoever claims a vertex delivers both with a single put instead of two scattered 4-byte ones
// -- half the partial-sector writes of a level.  The caller's separate level / parent arrays are filled from
// the records when the search is over.
__device__ __forceinline__ uint64_t bfs_pl(uint32_t parent, int32_t level)
{
    return ((uint64_t)(uint32_t)level << 32) | parent;
}
__device__ __forceinline__ uint64_t *bfs_pl_of(const Ctx &c, const BfsState &s, uint32_t pe)
{
    return (uint64_t *)ptr(c, s.pl_off, pe);
}

// Once per graph: the adjacency in the library's numbering.  Vertices are ranked by degree (largest first, ties by
// the caller's number) and rank r becomes local vertex r / npes of PE r mod npes -- still a 1D partition, every PE
// holding an equal share of every degree class, with the vertices that most edges point to at the start of every
// PE's block (that is where the top-down kernels' LDS filter looks, see HubFilter).  A wave copies one row at a
// time, in the caller's neighbour order, translating the neighbours.
// A neighbour that is no vertex (>= nverts_orig) is reported through *bad (host-visible; the row's own vertex is
// written in its place, so nothing downstream leaves its arrays) and shmem_bfs_create refuses the graph.
// Within a row the neighbours are put into four classes by their rank -- the best-connected 1/1024 of the
// vertices first, then those up to 1/64, up to 1/8, and the rest -- each class in the caller's order: a bottom-up
// level scans a row until it meets a frontier vertex, and the well-connected neighbours are the likeliest to be
// in the frontier; top-down, neighbouring lanes then probe bits that lie close together.
__global__ __launch_bounds__(256) void k_bfs_relabel(uint32_t nint, uint32_t nverts_orig, uint32_t vpp, const uint32_t *__restrict__ to_orig,
                                                     const uint32_t *__restrict__ to_int, const uint64_t *__restrict__ row_orig,
                                                     const uint32_t *__restrict__ nbr_orig, const uint64_t *__restrict__ row_int,
                                                     uint32_t *__restrict__ nbr_int, uint64_t *bad)
{
    const uint32_t lane = threadIdx.x & 63;
    const uint64_t wave = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6, waves = ((uint64_t)gridDim.x * blockDim.x) >> 6;
    const uint32_t lim0 = max(1u, vpp >> 10), lim1 = max(1u, vpp >> 6), lim2 = max(1u, vpp >> 3);
    for (uint64_t i = wave; i < nint; i += waves) {
        const uint32_t o = to_orig[i];
        if (o == SHMEM_BFS_NONE) continue;
        const uint64_t src = row_orig[o], dst = row_int[i], deg = row_int[i + 1] - dst;
        auto fetch = [&](uint64_t e, uint32_t &t, uint32_t &cls) {       // neighbour e of the row in the library's numbering, its class
            const uint32_t u = nbr_orig[src + e];
            if (u >= nverts_orig) __hip_atomic_store(bad, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            t = u < nverts_orig ? to_int[u] : (uint32_t)i;
            const uint32_t l = t % vpp;
            cls = l < lim0 ? 0u : l < lim1 ? 1u : l < lim2 ? 2u : 3u;
        };
        uint64_t at[4] = {0, 0, 0, 0};                                   // pass 1: how many of each class
        for (uint64_t e0 = 0; e0 < deg; e0 += 64) {
            uint32_t t = 0, cls = 4;
            if (e0 + lane < deg) fetch(e0 + lane, t, cls);
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k) at[k] += (uint64_t)__builtin_popcountll(ballot(cls == k));
        }
        at[3] = at[0] + at[1] + at[2]; at[2] = at[0] + at[1]; at[1] = at[0]; at[0] = 0;   // -> first place of each class
        for (uint64_t e0 = 0; e0 < deg; e0 += 64) {                      // pass 2: every neighbour to its place
            uint32_t t = 0, cls = 4;
            if (e0 + lane < deg) fetch(e0 + lane, t, cls);
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k) {
                const uint64_t m = ballot(cls == k);
                if (cls == k) nbr_int[dst + at[k] + rank_in(m)] = t;
                at[k] += (uint64_t)__builtin_popcountll(m);
            }
        }
    }
}

// Neighbour entries between the library's vertex number (owner * vpp + local) and the vertex's degree rank
// (local * npes + owner), in place: around the sort of the rows by rank.
__global__ __launch_bounds__(256) void k_bfs_rekey(uint32_t *nbr, uint64_t nnz, uint32_t vpp, uint32_t npes, int to_rank)
{
    const uint64_t size = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t e = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; e < nnz; e += size) {
        const uint32_t x = nbr[e];
        nbr[e] = to_rank ? (x % vpp) * npes + x / vpp : (x % npes) * vpp + x / npes;
    }
}

// Every owner clears its slice; the root's owner seeds the search.
// `prev_has_root`: the snapshot of the bitmap "as of the previous level" starts with the root in it (searches
// that derive a level's frontier bitmap level by level).  `make_front` (direction-optimising modes): level 0's
// frontier bitmap, the root alone, and its row length as the first degree sum.  The root's row length also goes
// to `host_root_deg` (GPU-mapped host memory).
__global__ __launch_bounds__(256) void k_bfs_init(Ctx c, BfsState s, uint32_t root, int prev_has_root, int make_front,
                                                  uint64_t *host_root_deg)
{
    const uint32_t pe = blockIdx.x / s.wgs_per_pe, wg = blockIdx.x % s.wgs_per_pe;
    const uint64_t rank = (uint64_t)wg * blockDim.x + threadIdx.x, size = (uint64_t)s.wgs_per_pe * blockDim.x;
    const uint32_t ro = bfs_owner(s, root), rl = root - ro * s.vpp;
    uint64_t *bm = (uint64_t *)ptr(c, s.bitmap_off, pe);
    uint64_t *pl = bfs_pl_of(c, s, pe);
    for (uint64_t w = rank; w < s.words; w += size)
        bm[w] = (pe == ro && w == bfs_vis_word(s, rl >> 6)) ? 1ull << (rl & 63) : 0ull;
    uint64_t *flt = (uint64_t *)ptr(c, s.filter_off, pe);
    for (uint64_t w = rank; w < s.words * NXCD; w += size) flt[w] = 0;
    uint64_t *prev = (uint64_t *)ptr(c, s.prev_off, pe);
    for (uint64_t w = rank; w < s.words; w += size)
        prev[w] = (prev_has_root && pe == ro && w == bfs_vis_word(s, rl >> 6)) ? 1ull << (rl & 63) : 0ull;   // laid out like the claim bitmap
    if (make_front) {
        uint64_t *front = (uint64_t *)ptr(c, s.front_off, pe);
        for (uint64_t w = rank; w < s.words; w += size) front[w] = (pe == ro && w == (rl >> 6)) ? 1ull << (rl & 63) : 0ull;
    }
    // The (parent, level) records are NOT cleared (8 bytes per vertex, more than everything else here together):
    // a record means something only while its vertex's bit is set in the bitmap, and every reader looks there first.
    if (rank == 0) {
        if (pe == ro) pl[rl] = bfs_pl(root, 0);
        uint64_t *t = bfs_tails(c, s, pe);
        t[T_TAIL0 + 0] = pe == ro ? 1 : 0; t[T_TAIL0 + 1] = 0; t[T_TAIL0 + 2] = 0;
        t[T_NBIG] = 0; t[T_NTASKS] = 0; t[T_ARRIVE] = 0; t[T_DEG_EXPANDED] = 0; t[T_DEG_FOUND] = 0; t[T_FILL] = 0;
        t[T_CLAIM_EXPAND] = 0; t[T_CLAIM_BIG] = 0;
        if (pe == ro) {
            ((uint32_t *)ptr(c, s.queue_off[0], pe))[0] = root;
            const uint64_t deg = s.row_off[root + 1] - s.row_off[root];
            if (make_front) t[T_DEG_FOUND] = deg;
            host_root_deg[0] = deg;
        }
        if (pe == 0) c.scratch[W_WORK + 4] = 0;   // arrival count of the level-end kernel
    }
}

// ---------------------------------------------------------------------------
// Per-wave staging of claimed vertices, one small buffer per owner in LDS.
// A full block of STAGE_BLOCK is written to the owner's queue with ONE fetch_add
// on its tail and one coalesced 256-byte put; the remainder goes out at kernel end
// (bfs_flush_workgroup).
struct Stage {
    uint32_t *cnt;   // [STAGE_PES]
    uint32_t *buf;   // [STAGE_PES][STAGE_CAP]
};

template <bool STAGED>
__device__ __forceinline__ void bfs_enqueue(const Ctx &c, const BfsState &s, const Stage &st, uint32_t L, bool won,
                                            uint32_t o, uint32_t v)
{
    uint64_t m = ballot(won);
    if (!m) return;
    const uint32_t lane = lane_id();
    if (STAGED) {
        // Every winner takes its place in its owner's staging buffer with a returning LDS add on the
        // wave's counter for that owner (lanes with the same owner are served one after the other by
        // the LDS itself) -- no loop over the owners present in the wave, which with two dozen winners
        // per chunk on a heavy level was half of a chunk's time.  A counter holds at most
        // STAGE_BLOCK - 1 between calls and grows by at most 64 here, so it stays below STAGE_CAP.
        if (won) {
            const uint32_t pos = __hip_atomic_fetch_add(&st.cnt[o], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
            st.buf[o * STAGE_CAP + pos] = v;
        }
        __builtin_amdgcn_wave_barrier();
        const uint32_t cn_l = lane < (uint32_t)c.npes ? st.cnt[lane] : 0;          // npes <= STAGE_PES <= 64
        uint64_t full = ballot(cn_l >= STAGE_BLOCK);
        while (full) {                                                             // rare: a block of 64 leaves
            const uint32_t ol = (uint32_t)__builtin_ctzll(full);
            full &= full - 1;
            const uint32_t cn = bcast32(cn_l, ol);
            uint32_t *buf = st.buf + ol * STAGE_CAP;
            uint32_t *queue = (uint32_t *)ptr(c, s.queue_off[(L + 1) & 1], ol);
            uint64_t base = 0;
            if (lane == 0) base = atomic_fetch_add(bfs_tails(c, s, ol) + T_TAIL0 + (L + 1) % 3, (uint64_t)STAGE_BLOCK);
            base = bcast64(base, 0);
            if (lane < STAGE_BLOCK) __builtin_nontemporal_store(buf[lane], queue + base + lane);   // put: one full block
            const uint32_t rest = cn - STAGE_BLOCK;
            const uint32_t moved = lane < rest ? buf[STAGE_BLOCK + lane] : 0;
            __builtin_amdgcn_wave_barrier();
            if (lane < rest) buf[lane] = moved;
            if (lane == 0) st.cnt[ol] = rest;
            __builtin_amdgcn_wave_barrier();
        }
    } else {
        while (m) {
            const uint32_t leader = (uint32_t)__builtin_ctzll(m);
            const uint32_t ol = bcast32(o, leader);
            const uint64_t grp = ballot(won && o == ol);
            const uint32_t n = (uint32_t)__builtin_popcountll(grp);
            uint32_t *queue = (uint32_t *)ptr(c, s.queue_off[(L + 1) & 1], ol);
            uint64_t *tail = bfs_tails(c, s, ol) + T_TAIL0 + (L + 1) % 3;
            uint64_t base = 0;
            if (lane == leader) base = atomic_fetch_add(tail, (uint64_t)n);
            base = bcast64(base, leader);
            if (won && o == ol) queue[base + rank_in(grp)] = v;       // put v
            m &= ~grp;
        }
    }
}

// Probe EPL neighbours per lane (v[k] of frontier vertex u[k]; inactive slots
// only take part in the wave-wide steps).
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
template <uint32_t EPL>
struct Probe {
    uint32_t o[EPL], l[EPL];
    uint64_t *f[EPL];
    uint64_t known[EPL];
};

// first half: owner, local index and the read of this die's bitmap copy (EPL probes in flight).
// Every slot holds a valid vertex (an inactive slot repeats an edge of the batch) and is probed whether
// or not it is active: with exactly EPL loads per call the compiler can wait for the probes alone
// later on; loads under a condition make it wait for everything outstanding, the neighbour loads of
// the next chunk included.
template <uint32_t EPL>
__device__ __forceinline__ void bfs_probe_issue(const Ctx &c, const BfsState &s, uint32_t xcd, Probe<EPL> &p,
                                                const uint32_t (&v)[EPL])
{
#pragma unroll
    for (uint32_t k = 0; k < EPL; ++k) {
        p.o[k] = bfs_owner(s, v[k]);
        p.l[k] = v[k] - p.o[k] * s.vpp;
        p.f[k] = (uint64_t *)ptr(c, s.filter_off, p.o[k]) + (uint64_t)xcd * s.words + (p.l[k] >> 6);
        p.known[k] = *p.f[k];
    }
}

// second half, part one: claim what is not known to be claimed and wait for the outcome.  All claims of
// the chunk are issued before the first result is used: a fetch_or resolves at the memory side, so one
// round trip covers EPL of them.  Returns false when no lane of the wave had anything to claim (the
// common case late in a search).
template <uint32_t EPL>
struct Claim {
    bool need[EPL], won[EPL];
    uint64_t old[EPL];
};

template <uint32_t EPL>
__device__ __forceinline__ bool bfs_claim(const Ctx &c, const BfsState &s, const Probe<EPL> &p, const bool (&act)[EPL], Claim<EPL> &cl)
{
    bool any = false;
#pragma unroll
    for (uint32_t k = 0; k < EPL; ++k) {
        cl.need[k] = act[k] && !(p.known[k] & (1ull << (p.l[k] & 63)));
        any |= cl.need[k];
        cl.won[k] = false;
        cl.old[k] = 0;
    }
    if (!ballot(any)) return false;
#pragma unroll
    for (uint32_t k = 0; k < EPL; ++k)
        if (cl.need[k])
            cl.old[k] = atomic_fetch_or((uint64_t *)ptr(c, s.bitmap_off, p.o[k]) + bfs_vis_word(s, p.l[k] >> 6), 1ull << (p.l[k] & 63));   // the claim
#pragma unroll
    for (uint32_t k = 0; k < EPL; ++k) cl.won[k] = cl.need[k] && !(cl.old[k] & (1ull << (p.l[k] & 63)));
    return true;
}

// second half, part two: update this die's bitmap copy, deliver parent / level, enqueue the winners.
// (v, u) are the chunk's vertices; the caller has moved on to the next chunk's registers by now.
template <bool STAGED, uint32_t EPL>
__device__ __forceinline__ void bfs_deliver(const Ctx &c, const BfsState &s, const Stage &st, uint32_t L, const Probe<EPL> &p,
                                            const Claim<EPL> &cl, const uint32_t (&v)[EPL], const uint32_t (&u)[EPL])
{
    // the queue first: a full staging block waits for its fetch_add on the owner's tail, and that wait
    // should not have the scattered stores below in front of it
#pragma unroll
    for (uint32_t k = 0; k < EPL; ++k) bfs_enqueue<STAGED>(c, s, st, L, cl.won[k], p.o[k], v[k]);
#pragma unroll
    for (uint32_t k = 0; k < EPL; ++k) {
        if (cl.need[k]) {
            *p.f[k] = p.known[k] | cl.old[k] | (1ull << (p.l[k] & 63));   // everything the fetch_or showed to be claimed
            if (cl.won[k]) {
                // put (parent, level): one streaming 8-byte store, so the scattered lines do not push the
                // bitmap copies out of L2
                __builtin_nontemporal_store(bfs_pl(u[k], (int32_t)(L + 1)), bfs_pl_of(c, s, p.o[k]) + p.l[k]);
            }
        }
    }
}

// LDS of one workgroup (4 waves)
struct BfsLds {
    uint32_t cnt[4][STAGE_PES];
    uint32_t buf[4][STAGE_PES * STAGE_CAP];
    uint32_t pre[4][64];
    uint32_t u[4][64];
    uint64_t r0[4][64];
    uint64_t base[STAGE_PES];    // end of the kernel: where the workgroup's leftovers go in every owner's queue
};

// What is left in the four waves' staging buffers when the kernel ends goes out per WORKGROUP: one fetch_add per
// owner for all four waves (the lanes of wave 0 issue them side by side), then every wave writes its entries behind
// those of the waves before it.  A wave flushing on its own made 16 dependent round trips, and a launch put
// 4096 adds on each of the 16 tails, which the memory takes one at a time: on the level that expands a few dozen
// hubs -- one chunk per wave, every wave a few winners for every owner -- that was most of the kernel's time.
// Every thread of the workgroup must call it.
template <bool STAGED>
__device__ __forceinline__ void bfs_flush_workgroup(const Ctx &c, const BfsState &s, BfsLds &lds, uint32_t L)
{
    if (!STAGED) return;
    const uint32_t lane = lane_id(), wave = threadIdx.x >> 6;
    __syncthreads();
    if (wave == 0 && lane < (uint32_t)c.npes) {
        const uint32_t tot = lds.cnt[0][lane] + lds.cnt[1][lane] + lds.cnt[2][lane] + lds.cnt[3][lane];
        lds.base[lane] = tot ? atomic_fetch_add(bfs_tails(c, s, lane) + T_TAIL0 + (L + 1) % 3, (uint64_t)tot) : 0;
    }
    __syncthreads();
    for (uint32_t o = 0; o < (uint32_t)c.npes; ++o) {
        const uint32_t cn = lds.cnt[wave][o];
        if (cn == 0) continue;
        uint64_t at = lds.base[o];
        for (uint32_t w = 0; w < wave; ++w) at += lds.cnt[w][o];
        if (lane < cn) ((uint32_t *)ptr(c, s.queue_off[(L + 1) & 1], o))[at + lane] = lds.buf[wave][o * STAGE_CAP + lane];
    }
}

// How the top-down kernels of a level share their work inside a PE: it is CLAIMED, not dealt.  A wave takes its
// first batch (run) by its number and every further one from a counter of the PE when it has finished the one
// before (nothing is held in reserve: what a wave holds nobody else can take over at the end), so that the slow
// waves of a PE take less and its fast ones more.  Per-wave timestamps showed why: the chip places the workgroups
// of a launch in order, four to a compute unit, and the waves run at very different speeds (with equal shares
// the waves of a heavy level finished between 0.15 and 1.63 ms).  The PE of a workgroup stays b / wgs_per_pe:
// dealing the workgroups of every vintage and die to every PE evened the PEs out but made every level slower.
//
// Expand level L: short rows packed, long rows set aside.
template <bool STAGED>
__global__ __launch_bounds__(256) void k_bfs_expand(Ctx c, BfsState s, uint32_t L)
{
    constexpr uint32_t EPL = EPL_SHORT;
    __shared__ BfsLds lds;
    const uint32_t pe = blockIdx.x / s.wgs_per_pe, wg = blockIdx.x % s.wgs_per_pe;
    const uint32_t lane = threadIdx.x & 63, wpw = blockDim.x >> 6;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: keeps wave state in SGPRs
    const uint64_t team_waves = (uint64_t)s.wgs_per_pe * wpw, my_wave = (uint64_t)wg * wpw + wave;
    const uint32_t xcd = xcd_id();
    const Stage st{lds.cnt[wave], lds.buf[wave]};
    if (STAGED && lane < STAGE_PES) st.cnt[lane] = 0;
    __builtin_amdgcn_wave_barrier();
    uint32_t *pre = lds.pre[wave], *su = lds.u[wave];
    uint64_t *sr0 = lds.r0[wave];
    uint64_t *tails = bfs_tails(c, s, pe);
    const uint64_t cnt = tails[T_TAIL0 + L % 3];
    const uint32_t *queue = (const uint32_t *)ptr(c, s.queue_off[L & 1], pe);
    uint32_t *big = (uint32_t *)ptr(c, s.big_off, pe);
    uint64_t degsum = 0;
    // a batch is 64 frontier vertices, or 16 while the frontier is short (a short frontier is the hubs: 64 of
    // them are a millisecond of edges, and a PE's waves would have one batch each, or two)
    const uint32_t bs = cnt >= team_waves * 64 * 4 ? 64u : 16u;
    const uint64_t nbatch = (cnt + bs - 1) / bs;
    uint64_t batch = my_wave;                        // the first one by number, the others claimed (a round trip of a
    for (bool first = true;; first = false) {        // microsecond or two per batch of a hundred)
        if (!first) {
            uint64_t got = 0;
            if (lane == 0) got = atomic_fetch_add(tails + T_CLAIM_EXPAND, 1);
            batch = team_waves + bcast64(got, 0);
        }
        if (batch >= nbatch) break;
        const uint64_t base = batch * bs;
        const bool valid = lane < bs && base + lane < cnt;
        uint32_t u = 0, deg = 0;
        uint64_t r0 = 0;
        if (valid) {
            u = __builtin_nontemporal_load(queue + base + lane);
            r0 = __builtin_nontemporal_load(s.row_off + u);
            deg = (uint32_t)(__builtin_nontemporal_load(s.row_off + u + 1) - r0);
        }
        degsum += deg;
        const bool is_big = deg >= BIG_DEGREE;
        const uint64_t bm = ballot(is_big);
        if (bm) {                                   // long rows: one fetch_add reserves list slots for the wave
            uint64_t hb = 0;
            if (lane == 0) hb = atomic_fetch_add(tails + T_NBIG, (uint64_t)__builtin_popcountll(bm));
            hb = bcast64(hb, 0);
            if (is_big) big[hb + rank_in(bm)] = u;
        }
        // wave-wide inclusive prefix sum of the short rows' lengths
        const uint32_t small = is_big ? 0 : deg;
        uint32_t incl = small;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t t = __shfl_up(incl, d, 64);
            if (lane >= (uint32_t)d) incl += t;
        }
        const uint32_t total = bcast32(incl, 63);
        if (total == 0) continue;
        pre[lane] = incl - small; su[lane] = u; sr0[lane] = r0;
        __builtin_amdgcn_wave_barrier();
        // edges e0 .. e0 + 64*EPL of the batch: owning row by binary search over the prefix sums
        // (a slot beyond the batch's last edge repeats that edge, inactive: always EPL loads, all in bounds)
        auto fetch = [&](uint32_t e0, bool (&act)[EPL], uint32_t (&vv)[EPL], uint32_t (&uu)[EPL]) {
#pragma unroll
            for (uint32_t k = 0; k < EPL; ++k) {
                const uint32_t e_ = e0 + k * 64 + lane;
                act[k] = e_ < total;
                const uint32_t e = act[k] ? e_ : total - 1;
                uint32_t lo = 0;                     // largest i with pre[i] <= e
#pragma unroll
                for (int step = 32; step > 0; step >>= 1)
                    if (pre[lo + step] <= e) lo += step;
                uu[k] = su[lo];
                vv[k] = __builtin_nontemporal_load(s.nbr + sr0[lo] + (e - pre[lo]));
            }
        };
        bool act[EPL], nact[EPL];
        uint32_t vv[EPL], uu[EPL], nvv[EPL], nuu[EPL];
        fetch(0, act, vv, uu);
#pragma unroll
        for (uint32_t k = 0; k < EPL; ++k) asm volatile("" : : "v"(vv[k]));   // arrived before the loop is entered (see below)
        for (uint32_t e0 = 0; e0 < total; e0 += 64 * EPL) {
            Probe<EPL> pr;
            bfs_probe_issue(c, s, xcd, pr, vv);
            const bool more = e0 + 64 * EPL < total;
            fetch(more ? e0 + 64 * EPL : e0, nact, nvv, nuu);  // next neighbours travel while this chunk is probed (the last chunk asks for itself again)
            // The wait for the claims also sees the next neighbours arrive (they were requested earlier), so
            // the registers move on to the next chunk HERE, before this chunk's stores and queue traffic
            // go out: at the top of the loop nothing then has to wait for those to drain.  (The memory
            // counter is in order: waiting for a load issued before a varying number of stores means
            // waiting for all of them.)
            Claim<EPL> cl;
            const bool claimed = bfs_claim(c, s, pr, act, cl);
            uint32_t cv[EPL], cu[EPL];
#pragma unroll
            for (uint32_t k = 0; k < EPL; ++k) {
                asm volatile("" : : "v"(nvv[k]));    // the next neighbours are waited for here, not at the top of the loop
                cv[k] = vv[k]; cu[k] = uu[k]; act[k] = nact[k]; vv[k] = nvv[k]; uu[k] = nuu[k];
            }
            if (claimed) bfs_deliver<STAGED, EPL>(c, s, st, L, pr, cl, cv, cu);
        }
        __builtin_amdgcn_wave_barrier();
    }
    bfs_flush_workgroup<STAGED>(c, s, lds, L);
    // degree sum of this level's frontier -> traversed-edge count
    for (int off = 32; off > 0; off >>= 1) degsum += __shfl_down(degsum, off, 64);
    if (lane == 0 && degsum) atomic_fetch_add(tails + T_DEG_EXPANDED, degsum);
}

// Prefix sum over the long rows' segment counts of each PE (one workgroup per
// PE): scan[i] = first segment id of long row i, scan[nbig] = segments in total.
__global__ __launch_bounds__(1024) void k_bfs_bigscan(Ctx c, BfsState s)
{
    __shared__ uint32_t wsum[16];
    __shared__ uint32_t carry_s;
    const uint32_t pe = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint64_t *tails = bfs_tails(c, s, pe);
    const uint32_t nbig = (uint32_t)tails[T_NBIG];
    const uint32_t *big = (const uint32_t *)ptr(c, s.big_off, pe);
    uint32_t *scan = (uint32_t *)ptr(c, s.bigscan_off, pe);
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (uint32_t base = 0; base < nbig; base += blockDim.x) {
        const uint32_t i = base + threadIdx.x;
        uint32_t segs = 0;
        if (i < nbig) {
            const uint32_t u = big[i];
            segs = (uint32_t)((s.row_off[u + 1] - s.row_off[u] + SEG_EDGES - 1) / SEG_EDGES);
        }
        uint32_t incl = segs;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t t = __shfl_up(incl, d, 64);
            if (lane >= (uint32_t)d) incl += t;
        }
        if (lane == 63) wsum[wave] = incl;
        __syncthreads();
        uint32_t before = carry_s;
        for (uint32_t w = 0; w < wave; ++w) before += wsum[w];
        if (i < nbig) scan[i] = before + incl - segs;
        __syncthreads();
        if (threadIdx.x == blockDim.x - 1) carry_s = before + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) { scan[nbig] = carry_s; tails[T_NTASKS] = carry_s; }
}

// Long rows of level L, as 512-edge segments numbered through all the PE's long rows: a wave takes runs of
// up to BIG_RUN consecutive segments, the first by its number, the others claimed from a counter of the PE (see above
// k_bfs_expand).  Finding the row a run starts in is a search in the segment scan; its upper levels are a
// sample of the scan that every workgroup keeps in LDS, so a search costs two or three dependent reads of
// global memory instead of a dozen.
constexpr uint32_t BIG_RUN = 16;
constexpr uint32_t BIG_SAMPLES = 128;     // (with 512 the workgroup no longer fitted a compute unit four times)
template <bool STAGED>
__global__ __launch_bounds__(256) void k_bfs_big(Ctx c, BfsState s, uint32_t L)
{
    constexpr uint32_t EPL = EPL_LONG;
    __shared__ BfsLds lds;
    __shared__ uint32_t sample[BIG_SAMPLES];
    const uint32_t pe = blockIdx.x / s.wgs_per_pe, wg = blockIdx.x % s.wgs_per_pe;
    const uint32_t lane = threadIdx.x & 63, wpw = blockDim.x >> 6;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint64_t team_waves = (uint64_t)s.wgs_per_pe * wpw, my_wave = (uint64_t)wg * wpw + wave;
    uint64_t *tails = bfs_tails(c, s, pe);
    const uint32_t nbig = (uint32_t)tails[T_NBIG], ntasks = (uint32_t)tails[T_NTASKS];
    if (ntasks == 0) return;                         // the whole workgroup
    const uint32_t xcd = xcd_id();
    const Stage st{lds.cnt[wave], lds.buf[wave]};
    if (STAGED && lane < STAGE_PES) st.cnt[lane] = 0;
    const uint32_t *big = (const uint32_t *)ptr(c, s.big_off, pe);
    const uint32_t *scan = (const uint32_t *)ptr(c, s.bigscan_off, pe);
    // sample[j] = scan[j * stride]: first segment of every stride-th long row
    const uint32_t stride = (nbig + BIG_SAMPLES - 1) / BIG_SAMPLES, nsamples = (nbig + stride - 1) / stride;
    for (uint32_t j = threadIdx.x; j < nsamples; j += blockDim.x) sample[j] = scan[j * stride];
    __syncthreads();
    // runs of BIG_RUN segments; a level with few segments (a handful of hubs) is one equal run per wave, as claims
    // and searches would cost more than they even out
    const uint32_t R = ntasks >= team_waves * 4 * BIG_RUN ? BIG_RUN : (uint32_t)((ntasks + team_waves - 1) / team_waves);
    const uint64_t nruns = ((uint64_t)ntasks + R - 1) / R;
    uint64_t run = my_wave;
    for (bool first_run = true;; first_run = false) {
        if (!first_run) {
            uint64_t got = 0;
            if (lane == 0) got = atomic_fetch_add(tails + T_CLAIM_BIG, 1);
            run = team_waves + bcast64(got, 0);
        }
        if (run >= nruns) break;
        const uint32_t t0 = (uint32_t)(run * R), t1 = min(t0 + R, ntasks);
        uint32_t i;                                  // long row that holds segment t0: the last with scan[i] <= t0
        {
            uint32_t lo = 0, hi = nsamples;          // sample[lo] <= t0 < sample[hi] (sample[nsamples] = infinity)
            while (hi - lo > 1) {
                const uint32_t mid = (lo + hi) >> 1;
                if (sample[mid] <= t0) lo = mid; else hi = mid;
            }
            i = lo * stride;
            for (uint32_t up = min(i + stride, nbig); up - i > 1;) {
                const uint32_t mid = i + (up - i) / 2;
                if (scan[mid] <= t0) i = mid; else up = mid;
            }
        }
        uint32_t first = scan[i], next = scan[i + 1], u = big[i];
        uint64_t r0 = s.row_off[u], deg = s.row_off[u + 1] - r0;
        // neighbours of segment t (the row cursor only moves forward)
        auto fetch = [&](uint32_t t, bool (&act)[EPL], uint32_t (&vv)[EPL], uint32_t (&uu)[EPL]) {
            while (t >= next) {
                ++i; first = next; next = scan[i + 1]; u = big[i];
                r0 = s.row_off[u]; deg = s.row_off[u + 1] - r0;
            }
            const uint64_t e0 = (uint64_t)(t - first) * SEG_EDGES;
#pragma unroll
            for (uint32_t k = 0; k < EPL; ++k) {
                const uint64_t e = e0 + k * 64 + lane;
                act[k] = e < deg;
                uu[k] = u;
                vv[k] = __builtin_nontemporal_load(s.nbr + r0 + (act[k] ? e : deg - 1));   // always a load, always in bounds
            }
        };
        bool act[EPL], nact[EPL];
        uint32_t vv[EPL], uu[EPL], nvv[EPL], nuu[EPL];
        fetch(t0, act, vv, uu);
#pragma unroll
        for (uint32_t k = 0; k < EPL; ++k) asm volatile("" : : "v"(vv[k]));   // arrived before the loop is entered
        for (uint32_t t = t0; t < t1; ++t) {
            Probe<EPL> pr;
            bfs_probe_issue(c, s, xcd, pr, vv);
            const bool more = t + 1 < t1;
            fetch(more ? t + 1 : t, nact, nvv, nuu);         // next segment travels while this one is probed (the last asks for itself again)
            Claim<EPL> cl;
            const bool claimed = bfs_claim(c, s, pr, act, cl);           // (as in k_bfs_expand)
            uint32_t cv[EPL], cu[EPL];
#pragma unroll
            for (uint32_t k = 0; k < EPL; ++k) {
                asm volatile("" : : "v"(nvv[k]));    // the next neighbours are waited for here, not at the top of the loop
                cv[k] = vv[k]; cu[k] = uu[k]; act[k] = nact[k]; vv[k] = nvv[k]; uu[k] = nuu[k];
            }
            if (claimed) bfs_deliver<STAGED, EPL>(c, s, st, L, pr, cl, cv, cu);
        }
    }
    bfs_flush_workgroup<STAGED>(c, s, lds, L);
}

// ---------------------------------------------------------------------------
// Direction-optimising levels (optional).  A bottom-up level turns the search
// round: every owner scans ITS OWN unvisited vertices and looks for a neighbour
// in the current frontier with one-sided gets of the frontier bitmap; the
// claim, parent, level and queue entry are then local (owner computes, no
// atomics on the bitmap).  It examines far fewer edges than top-down once the
// frontier holds most of the remaining edges.

// Once per graph: bit l of the owner's `linked` bitmap = local vertex l has a non-empty row.
__global__ __launch_bounds__(256) void k_bfs_mark_linked(Ctx c, BfsState s)
{
    const uint32_t pe = blockIdx.x / s.wgs_per_pe, wg = blockIdx.x % s.wgs_per_pe;
    const uint32_t lane = threadIdx.x & 63, wpw = blockDim.x >> 6, wave = threadIdx.x >> 6;
    const uint64_t team_waves = (uint64_t)s.wgs_per_pe * wpw, my_wave = (uint64_t)wg * wpw + wave;
    const uint64_t first = (uint64_t)pe * s.vpp;
    const uint64_t count = first >= s.nverts ? 0 : (s.nverts - first < s.vpp ? s.nverts - first : s.vpp);
    uint64_t *linked = (uint64_t *)ptr(c, s.linked_off, pe);
    for (uint64_t w = my_wave; w < s.words; w += team_waves) {
        const uint64_t l = w * 64 + lane;
        const bool has = l < count && s.row_off[first + l + 1] > s.row_off[first + l];
        const uint64_t m = ballot(has);
        if (lane == 0) linked[w] = m;
    }
}

// is u in the current frontier?  (an 8-byte get from u's owner)
__device__ __forceinline__ bool bfs_in_front(const Ctx &c, const BfsState &s, uint32_t u)
{
    const uint32_t o = bfs_owner(s, u), lu = u - o * s.vpp;
    return (((const uint64_t *)ptr(c, s.front_off, o))[lu >> 6] >> (lu & 63)) & 1;
}

constexpr uint32_t BU_LANE_EDGES = 16;  // neighbours a lane scans on its own before the wave helps
constexpr uint32_t BU_BATCH = 4;        // ... this many at a time

// Bottom-up level L -> L+1.  A wave owns one bitmap word (64 consecutive local
// vertices, lane = bit) at a time.
__global__ __launch_bounds__(256) void k_bfs_bottomup(Ctx c, BfsState s, uint32_t L)
{
    const uint32_t pe = blockIdx.x / s.wgs_per_pe, wg = blockIdx.x % s.wgs_per_pe;
    const uint32_t lane = threadIdx.x & 63, wpw = blockDim.x >> 6;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint64_t team_waves = (uint64_t)s.wgs_per_pe * wpw, my_wave = (uint64_t)wg * wpw + wave;
    const uint64_t first = (uint64_t)pe * s.vpp;
    if (first >= s.nverts) return;
    const uint64_t count = s.nverts - first < s.vpp ? s.nverts - first : s.vpp;
    uint64_t *vis = (uint64_t *)ptr(c, s.bitmap_off, pe);
    const uint64_t *linked = (const uint64_t *)ptr(c, s.linked_off, pe);
    uint64_t *pl = bfs_pl_of(c, s, pe);
    uint64_t *tail = bfs_tails(c, s, pe) + T_TAIL0 + (L + 1) % 3;
    uint64_t mf = 0;
    uint32_t nfound = 0;   // wave-uniform
    for (uint64_t w = my_wave; w * 64 < count; w += team_waves) {
        const uint64_t vw = bfs_vis_word(s, w);
        const uint64_t visw = vis[vw];
        const uint64_t todo = ~visw & linked[w];         // unvisited vertices that have neighbours
        if (todo == 0) continue;
        const uint64_t l = w * 64 + lane;
        uint32_t par = SHMEM_BFS_NONE, deg = 0;
        uint64_t r0 = 0;
        if ((todo >> lane) & 1) {
            r0 = s.row_off[first + l];
            deg = (uint32_t)(s.row_off[first + l + 1] - r0);
            const uint32_t own = deg < BU_LANE_EDGES ? deg : BU_LANE_EDGES;   // the lane's own share of the row
            // the first neighbour alone (the best-connected of the row: the likeliest to be in the frontier) ...
            if (own) {
                const uint32_t u0 = s.nbr[r0];
                if (bfs_in_front(c, s, u0)) par = u0;
            }
            // ... then four neighbours and their four frontier words travel together; the first hit in row order wins
            for (uint32_t j = 1; j < own && par == SHMEM_BFS_NONE; j += BU_BATCH) {
                uint32_t u[BU_BATCH];
                bool in[BU_BATCH];
#pragma unroll
                for (uint32_t k = 0; k < BU_BATCH; ++k) u[k] = j + k < own ? s.nbr[r0 + j + k] : 0;
#pragma unroll
                for (uint32_t k = 0; k < BU_BATCH; ++k) in[k] = j + k < own && bfs_in_front(c, s, u[k]);
#pragma unroll
                for (uint32_t k = BU_BATCH; k-- > 0;) if (in[k]) par = u[k];
            }
        }
        // rows longer than a lane's share: the whole wave scans the rest, 64 neighbours at a time
        uint64_t longrows = ballot(par == SHMEM_BFS_NONE && deg > BU_LANE_EDGES);
        while (longrows) {
            const uint32_t j = (uint32_t)__builtin_ctzll(longrows);
            longrows &= longrows - 1;
            const uint32_t dj = bcast32(deg, j);
            const uint64_t rj = bcast64(r0, j);
            uint32_t hit = SHMEM_BFS_NONE;
            for (uint32_t e0 = BU_LANE_EDGES; e0 < dj && hit == SHMEM_BFS_NONE; e0 += 64) {
                const bool act = e0 + lane < dj;
                const uint32_t u = act ? s.nbr[rj + e0 + lane] : 0;
                const uint64_t hm = ballot(act && bfs_in_front(c, s, u));
                if (hm) hit = bcast32(u, (uint32_t)__builtin_ctzll(hm));
            }
            if (lane == j) par = hit;
        }
        const bool found = par != SHMEM_BFS_NONE;
        const uint64_t fm = ballot(found);
        if (fm == 0) continue;
        if (lane == 0) vis[vw] = visw | fm;              // this wave is the only writer of the word
        nfound += (uint32_t)__builtin_popcountll(fm);
        if (found) {
            pl[l] = bfs_pl(par, (int32_t)(L + 1));
            mf += deg;
        }
    }
    // The new frontier is only counted here (one add per wave; an add per bitmap word, thousands on
    // one address per PE, serialised for tens of microseconds).  Its queue is written by
    // k_bfs_fill_queue from the frontier bitmap if the next level turns out to run top-down.
    if (lane == 0 && nfound) atomic_fetch_add(tail, (uint64_t)nfound);
    for (int off = 32; off > 0; off >>= 1) mf += __shfl_down(mf, off, 64);
    if (lane == 0 && mf) atomic_fetch_add(bfs_tails(c, s, pe) + T_DEG_FOUND, mf);
}

// The owner's queue for level `next` written from its frontier bitmap (the bits set during the last level;
// k_bfs_level_end has built it): after a bottom-up level, which only counts its finds, before a top-down one;
// and before the top-down expansion of a LARGE frontier, whose queue then lists the vertices in ascending runs
// instead of in the order the claims arrived -- a batch of 64 frontier vertices reads neighbouring rows of the
// adjacency, which share their 128-byte lines, and its row offsets in a few coalesced requests.  A wave takes
// 64 consecutive words, one per lane, reserves room for all their bits with one add and writes the vertices.
__global__ __launch_bounds__(256) void k_bfs_fill_queue(Ctx c, BfsState s, uint32_t next)
{
    const uint32_t pe = blockIdx.x / s.wgs_per_pe, wg = blockIdx.x % s.wgs_per_pe;
    const uint32_t lane = threadIdx.x & 63, wpw = blockDim.x >> 6;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint64_t team_waves = (uint64_t)s.wgs_per_pe * wpw, my_wave = (uint64_t)wg * wpw + wave;
    const uint64_t *front = (const uint64_t *)ptr(c, s.front_off, pe);
    uint32_t *queue = (uint32_t *)ptr(c, s.queue_off[next & 1], pe);
    uint64_t *fill = bfs_tails(c, s, pe) + T_FILL;
    const uint64_t first = (uint64_t)pe * s.vpp;
    for (uint64_t w0 = my_wave * 64; w0 < s.words; w0 += team_waves * 64) {
        const uint64_t w = w0 + lane;
        uint64_t bits = w < s.words ? front[w] : 0;
        const uint32_t n = (uint32_t)__builtin_popcountll(bits);
        uint32_t incl = n;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t t = __shfl_up(incl, d, 64);
            if (lane >= (uint32_t)d) incl += t;
        }
        const uint32_t total = bcast32(incl, 63);
        if (total == 0) continue;
        uint64_t base = 0;
        if (lane == 0) base = atomic_fetch_add(fill, (uint64_t)total);
        base = bcast64(base, 0);
        // word by word, the whole wave writing the vertices of one word side by side (in the library's numbering the
        // best-connected vertices come first, so the words at the start of a block are full and the rest nearly
        // empty: a lane writing out its own word kept the wave busy for 64 rounds of scattered stores)
        uint64_t nonempty = ballot(n != 0);
        while (nonempty) {
            const uint32_t j = (uint32_t)__builtin_ctzll(nonempty);
            nonempty &= nonempty - 1;
            const uint64_t bj = bcast64(bits, j);
            const uint64_t at = base + bcast32(incl - n, j);
            if ((bj >> lane) & 1) queue[at + rank_in(bj)] = (uint32_t)(first + (w0 + j) * 64 + lane);
        }
    }
}

// Optional post-pass: canonical parents.  parent[v] = the smallest neighbour of v whose level is one
// less than v's (levels are unique, so this tree is too and can be compared vertex by vertex).  Every
// owner rewrites the parents of its own vertices; a neighbour's level is a 4-byte get from its owner.
constexpr uint32_t CANON_LANE_EDGES = 32;   // rows up to this long are scanned by one lane

__device__ __forceinline__ int32_t bfs_level_of(const Ctx &c, const BfsState &s, uint32_t u)
{
    const uint32_t o = bfs_owner(s, u);
    return ((const int32_t *)ptr(c, s.pl_off, o))[2 * (uint64_t)(u - o * s.vpp) + 1];    // the high word of the record
}

__global__ __launch_bounds__(256) void k_bfs_canonical(Ctx c, BfsState s)
{
    const uint32_t pe = blockIdx.x / s.wgs_per_pe, wg = blockIdx.x % s.wgs_per_pe;
    const uint32_t lane = threadIdx.x & 63, wpw = blockDim.x >> 6;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint64_t team_waves = (uint64_t)s.wgs_per_pe * wpw, my_wave = (uint64_t)wg * wpw + wave;
    const uint64_t first = (uint64_t)pe * s.vpp;
    if (first >= s.nverts) return;
    const uint64_t count = s.nverts - first < s.vpp ? s.nverts - first : s.vpp;
    uint64_t *pl = bfs_pl_of(c, s, pe);
    const uint64_t *vis = (const uint64_t *)ptr(c, s.bitmap_off, pe);
    for (uint64_t w = my_wave; w * 64 < count; w += team_waves) {
        const uint64_t l = w * 64 + lane;
        const bool reached = l < count && ((vis[bfs_vis_word(s, w)] >> lane) & 1);     // an unreached vertex's record is stale
        const int32_t lvl = reached ? (int32_t)(pl[l] >> 32) : -1;
        const bool need = lvl > 0;                       // reached and not the root
        // "smallest" is by the CALLER's numbers (bo), what is stored is the library's (best)
        uint32_t best = SHMEM_BFS_NONE, bo = SHMEM_BFS_NONE, deg = 0;
        uint64_t r0 = 0;
        if (need) {
            r0 = s.row_off[first + l];
            deg = (uint32_t)(s.row_off[first + l + 1] - r0);
            if (deg <= CANON_LANE_EDGES)
                for (uint32_t j = 0; j < deg; ++j) {
                    const uint32_t u = s.nbr[r0 + j], uo = s.to_orig[u];
                    if (bfs_level_of(c, s, u) == lvl - 1 && uo < bo) { bo = uo; best = u; }
                }
        }
        uint64_t longrows = ballot(need && deg > CANON_LANE_EDGES);   // the wave scans these together
        while (longrows) {
            const uint32_t j = (uint32_t)__builtin_ctzll(longrows);
            longrows &= longrows - 1;
            const uint32_t dj = bcast32(deg, j);
            const uint64_t rj = bcast64(r0, j);
            const int32_t lj = (int32_t)bcast32((uint32_t)lvl, j);
            uint64_t mn = ~0ull;                                      // (caller's number, library's number)
            for (uint32_t e0 = 0; e0 < dj; e0 += 64) {
                if (e0 + lane < dj) {
                    const uint32_t u = s.nbr[rj + e0 + lane];
                    if (bfs_level_of(c, s, u) == lj - 1) mn = min(mn, ((uint64_t)s.to_orig[u] << 32) | u);
                }
            }
            for (int off = 32; off > 0; off >>= 1) {
                const uint64_t other = ((uint64_t)(uint32_t)__shfl_xor((int)(uint32_t)(mn >> 32), off, 64) << 32) |
                                       (uint32_t)__shfl_xor((int)(uint32_t)mn, off, 64);
                mn = min(mn, other);
            }
            if (lane == j) best = mn == ~0ull ? SHMEM_BFS_NONE : (uint32_t)mn;
        }
        if (need) ((uint32_t *)(pl + l))[0] = best;      // the low word of the record
    }
}

// End of a level in one launch: (optionally) the frontier bitmap of the level about to be expanded and
// the sum of its row lengths, then -- by whichever workgroup finishes last -- the level epilogue of
// level epilogue (total size of frontier `next`, reset of the long-row counters and of the count that
// level next+1 will fill) and the hand-over to the host: the three level counters go into GPU-mapped
// pinned memory, then a sequence number behind a system-scope release; the host polls the sequence word
// instead of paying for a copy and a stream synchronisation per level.  Nobody waits inside the kernel:
// every workgroup counts itself in, and only the one that finds all others counted goes on.
__global__ __launch_bounds__(256) void k_bfs_level_end(Ctx c, BfsState s, uint32_t next, int do_front, int do_degree,
                                                       uint64_t *host_counts, uint64_t seq)
{
    __shared__ bool last;
    const uint32_t teams_wgs = gridDim.x / (uint32_t)c.npes;           // workgroups per PE in this launch
    const uint32_t pe = blockIdx.x / teams_wgs, wg = blockIdx.x % teams_wgs;
    const uint64_t rank = (uint64_t)wg * blockDim.x + threadIdx.x, size = (uint64_t)teams_wgs * blockDim.x;
    if (do_front) {
        const uint64_t *vis = (const uint64_t *)ptr(c, s.bitmap_off, pe);
        uint64_t *front = (uint64_t *)ptr(c, s.front_off, pe), *prev = (uint64_t *)ptr(c, s.prev_off, pe);
        // vis and prev are walked as they lie (prev has the claim bitmap's layout); only the frontier word is
        // stored where its number says
        for (uint64_t q = rank; q < s.words; q += size) {
            const uint64_t v = vis[q];
            front[bfs_vis_word_at(s, q)] = v & ~prev[q];
            prev[q] = v;
        }
    }
    if (do_degree) {
        const uint64_t cnt = bfs_tails(c, s, pe)[T_TAIL0 + next % 3];
        const uint32_t *queue = (const uint32_t *)ptr(c, s.queue_off[next & 1], pe);
        uint64_t sum = 0;
        for (uint64_t k = rank; k < cnt; k += size) {
            const uint32_t u = queue[k];
            sum += s.row_off[u + 1] - s.row_off[u];
        }
        for (int off = 32; off > 0; off >>= 1) sum += __shfl_down(sum, off, 64);
        if ((threadIdx.x & 63) == 0 && sum) atomic_fetch_add(bfs_tails(c, s, pe) + T_DEG_FOUND, sum);
    }
    // Everything the last workgroup reads below is an atomically updated counter, and those resolve at
    // the memory side: each wave's adds are complete (workgroup-scope release = wait for their
    // acknowledgement) before thread 0 counts the workgroup in, so no cache write-back or invalidate is
    // needed here; the plain stores above are for the next kernel and leave with this one's end.
    wg_release();
    if (threadIdx.x == 0) {
        // two stages (per PE, then across PEs): arrivals on one word serialise at the memory side
        last = false;
        uint64_t *mine = bfs_tails(c, s, pe) + T_ARRIVE;
        if (atomic_fetch_add(mine, 1) == teams_wgs - 1) {
            __hip_atomic_store(mine, 0ull, __ATOMIC_RELAXED, SHMEMX_AGENT);                     // all of this PE have arrived
            last = atomic_fetch_add(&c.scratch[W_WORK + 4], 1) == (uint64_t)c.npes - 1;
            if (last) __hip_atomic_store(&c.scratch[W_WORK + 4], 0ull, __ATOMIC_RELAXED, SHMEMX_AGENT);
        }
    }
    __syncthreads();
    if (!last || threadIdx.x >= 64) return;
    uint64_t total = 0, expanded = 0, found = 0;
    for (uint32_t q = threadIdx.x; q < (uint32_t)c.npes; q += 64) {
        uint64_t *t = bfs_tails(c, s, q);
        total += __hip_atomic_load(&t[T_TAIL0 + next % 3], __ATOMIC_RELAXED, SHMEMX_AGENT);
        expanded += __hip_atomic_load(&t[T_DEG_EXPANDED], __ATOMIC_RELAXED, SHMEMX_AGENT);
        found += __hip_atomic_load(&t[T_DEG_FOUND], __ATOMIC_RELAXED, SHMEMX_AGENT);
        t[T_TAIL0 + (next + 1) % 3] = 0;
        t[T_NBIG] = 0; t[T_NTASKS] = 0; t[T_FILL] = 0; t[T_CLAIM_EXPAND] = 0; t[T_CLAIM_BIG] = 0;
    }
    for (int off = 32; off > 0; off >>= 1) {
        total += __shfl_down(total, off, 64);
        expanded += __shfl_down(expanded, off, 64);
        found += __shfl_down(found, off, 64);
    }
    if (threadIdx.x == 0) {
        c.scratch[W_WORK] = total;
        host_counts[0] = total;
        host_counts[1] = expanded;
        host_counts[2] = found;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "");
        __hip_atomic_store(host_counts + 3, seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

// The (parent, level) records go into the caller's flat level / parent arrays, in the caller's numbering: thread
// o looks up where vertex o lives (to_int) and translates the parent it finds there (to_orig).
__global__ __launch_bounds__(256) void k_bfs_gather(Ctx c, BfsState s, uint32_t nverts_orig, const uint32_t *__restrict__ to_int,
                                                    int32_t *level, uint32_t *parent)
{
    const uint64_t rank = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x, size = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t o = rank; o < nverts_orig; o += size) {
        const uint32_t i = to_int[o], pe = bfs_owner(s, i), l = i - pe * s.vpp;
        const bool reached = (((const uint64_t *)ptr(c, s.bitmap_off, pe))[bfs_vis_word(s, l >> 6)] >> (l & 63)) & 1;
        const uint64_t rec = reached ? __builtin_nontemporal_load(bfs_pl_of(c, s, pe) + l) : bfs_pl(SHMEM_BFS_NONE, -1);
        const uint32_t par = (uint32_t)rec;
        if (level) __builtin_nontemporal_store((int32_t)(rec >> 32), level + o);
        if (parent) __builtin_nontemporal_store(par == SHMEM_BFS_NONE ? SHMEM_BFS_NONE : s.to_orig[par], parent + o);
    }
}

}  // namespace shmemx

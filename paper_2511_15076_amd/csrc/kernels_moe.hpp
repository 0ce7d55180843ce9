// MoE-shaped all-to-all in traffic shape: the low-latency dispatch and combine
// of Sec. IV-E ("Low-Latency Kernel Integration") at the message sizes of
// Sec. V-C (16 bytes of source-index metadata + the token; the token alone on
// the way back), on emulated PEs.  No quantisation, compression or weighted
// floating-point reduction: payloads are opaque bytes and the combine reduction
// is a wrapping sum of 32-bit words.
//
// Dispatch: every (token, expert) route is one message written straight into a
// receive slot at the expert's owner.  When all messages of one (sender,
// expert) pair are complete the sender delivers the pair's token count with a
// zero-byte put + SignalAdd (here: release, then a remote atomic add of
// count + 1 on signal le * npes + sender), so the count is only visible after
// the data.  Receivers poll their signals (readSignal), then pack what arrived
// per local expert: senders in ascending PE order, each sender's tokens in
// ascending token order.
// Combine: every expert output goes back to slot (token, top-k position) at the
// token's source PE; one flag signal per (expert, destination) pair follows the
// data; the destination waits for the flags of a token's experts and sums the
// copies.
//
// Work split, batches under 32 tokens per PE (latency-bound): workgroup w of a
// PE's team owns the experts e = w (mod team size) when sending and the local
// experts / tokens with the same residue when receiving, so one workgroup-level
// release covers all messages of a pair.  Larger batches (bandwidth-bound):
// messages are shared out half in fixed ranges, half in blocks claimed from a
// counter of the PE (moe_share), inside a workgroup piece by piece; a pair's
// count is then the sum of what several workgroups add after their releases.
// All workgroups of a launch are resident at once (the host checks the grid
// against the occupancy limit) and every workgroup finishes sending before it
// starts to wait, so the waits end; they are bounded besides.
#pragma once
#include "../../include/mi_shmem_gin.hpp"
#include "../../include/mi_shmemx.hpp"

namespace shmemx {


constexpr uint32_t MOE_MAX_EXPERTS = 1024;  // per-expert token masks live in LDS
constexpr uint32_t MOE_MAX_TOKENS = 128;    // two 64-bit mask words per expert
constexpr uint32_t MOE_MAX_TOPK = 64;       // one lane per top-k position
constexpr uint32_t MOE_MAX_PES = 256;
constexpr uint32_t MOE_META_BYTES = 16;
constexpr int MOE_THREADS = 512;              // eight waves per workgroup: more copies in flight per team
constexpr uint32_t MOE_BULK_TOKENS = 32;      // batches from this size on are balanced dynamically
constexpr uint32_t MOE_SEND_WAVES = 7;        // large batches: waves 0..6 move messages, the eighth claims work for them
constexpr uint32_t MOE_BLOCK = 1;             // messages per claim (see below)
constexpr uint32_t MOE_PARTS = 2;             // large batches: pieces of a message, each moved by one wave
// Measured at 128 tokens per PE: blocks of 2, 4 or 8 messages in 2 pieces were alike and 4 pieces per message cost 10 %
// while a wave moved one piece at a time; since a wave's next loads go out ahead of its stores a piece takes less, the
// last block a workgroup holds weighs more, and single messages are best: the combine, whose flags wait for the slowest
// workgroup of a PE, 75.7 -> 69.2 us at 128 tokens, 45.5 -> 40.7 at 64, 29.4 -> 27.3 at 32 (blocks of two: 73.5 / 42.8 /
// 29.6); the dispatch, which signals pair by pair, is unchanged.
// Whole messages as pieces (MOE_PARTS = 1) are excluded: the one measurement run with them produced no output for
// two minutes and was ended by its time limit, and reading the code has not shown why.
static_assert(MOE_PARTS >= 2, "see above");
constexpr uint32_t MOE_RANGES = 256;          // ranges of units one workgroup can take (blocks grow with the batch so that
                                              // one workgroup's list holds them all; at 512 the dispatch kernel's LDS was
                                              // 55,040 bytes as allocated and three workgroups did not fit a compute unit)
// per-PE control words, after the combine flags in the signal array
enum : uint32_t { MOE_CTL_COMBINES = 0, MOE_CTL_ARRIVALS = 1, MOE_CTL_SEND_CLAIM = 2, MOE_CTL_SEND_DONE = 3,
                  MOE_CTL_RECV_CLAIM = 4, MOE_CTL_RECV_DONE = 5, MOE_CTL_COMB_CLAIM = 6, MOE_CTL_COMB_DONE = 7, MOE_CTL_WORDS = 8 };

struct MoeState {
    uint32_t num_experts, epp, max_tokens, topk;
    uint64_t hidden, msg;    // token bytes (multiple of 16); dispatch message bytes = 16 + hidden
    uint64_t recv_off;       // symmetric: [epp][npes][max_tokens] dispatch messages
    uint64_t comb_off;       // symmetric: [max_tokens][topk] returned tokens
    GinState gin;            // signals [0, epp*npes): dispatch counts; then num_experts combine flags; then two
                             // words of the PE's own: combines completed, workgroups of the running combine that know it
};

struct MoeDispatchArgs {
    const uint8_t *x;        // [npes][max_tokens][hidden]
    const int32_t *topk;     // [npes][max_tokens][topk]
    const int32_t *ntok;     // [npes]
    uint8_t *recv_x;         // [npes][epp][npes*max_tokens][hidden]
    int32_t *recv_info;      // [npes][epp][npes*max_tokens][4]
    int32_t *recv_range;     // [npes][epp][npes][2]
    int32_t *recv_count;     // [npes][epp]
    uint32_t wgs_per_pe;
};

struct MoeCombineArgs {
    const uint8_t *expert_out;  // [npes][epp][npes*max_tokens][hidden]
    const int32_t *recv_info, *recv_range, *topk, *ntok;
    uint8_t *combined;          // [npes][max_tokens][hidden]
    uint32_t wgs_per_pe;
};

// Vectors [lo, lo + per) of a row of hvecs vectors that exist: 0 when the part starts at or beyond the end.
// In 64-bit signed arithmetic on purpose: the 32-bit unsigned form (lo < hvecs ? min(per, hvecs - lo) : 0)
// was compiled by hipcc 7.2, when an unpredicated variant of the copy below was tried next to it, into code
// that returned `per` for lo > hvecs (checked in isolation: same source, only this expression differing).
// A second hazard of that variant, whatever the compiler does: a copy that lets the lanes beyond the end
// repeat the LAST vector indexes vector count - 1, so it must never be entered with a count of 0 -- and parts
// with a count of 0 are exactly what messages split over more waves than they have vectors produce.
__device__ __forceinline__ uint32_t moe_part_vecs(uint32_t hvecs, uint32_t lo, uint32_t per)
{
    const int64_t rem = (int64_t)hvecs - (int64_t)lo;
    return rem <= 0 ? 0u : (uint32_t)(rem < (int64_t)per ? rem : (int64_t)per);
}

// One wave copies nv 16-byte vectors, eight loads per lane in flight.  THROUGH: the stores are written through
// (messages that a release and a signal follow: with nothing dirty left in the L2 that release is cheap -- one
// token per PE: combine 14.3 -> 12.6 us, eight: dispatch 25.5 -> 21.3, combine 24.4 -> 16.9); else streaming
// stores (rows packed for the caller).  CACHED: ordinary instead of streaming loads -- for the tokens a PE sends,
// each of which is read once per expert it goes to (top-k times, by different workgroups): 113.5 -> 108.4 us per dispatch
// of 128 tokens per PE.
template <bool THROUGH, bool CACHED = false>
__device__ __forceinline__ void wave_copy16(u32x4 *__restrict__ d, const u32x4 *__restrict__ s, uint32_t nv, uint32_t lane)
{
    constexpr int IF = 8;
    uint32_t i = lane;
    for (; i + (IF - 1) * 64 < nv; i += IF * 64) {
        u32x4 v[IF];
#pragma unroll
        for (int k = 0; k < IF; ++k) v[k] = CACHED ? s[i + 64 * k] : __builtin_nontemporal_load(s + i + 64 * k);
#pragma unroll
        for (int k = 0; k < IF; ++k) { if (THROUGH) store_through(v[k], d + i + 64 * k); else __builtin_nontemporal_store(v[k], d + i + 64 * k); }
    }
    u32x4 v[IF - 1];
#pragma unroll
    for (int k = 0; k < IF - 1; ++k) if (i + 64 * k < nv) v[k] = CACHED ? s[i + 64 * k] : __builtin_nontemporal_load(s + i + 64 * k);
#pragma unroll
    for (int k = 0; k < IF - 1; ++k) if (i + 64 * k < nv) { if (THROUGH) store_through(v[k], d + i + 64 * k); else __builtin_nontemporal_store(v[k], d + i + 64 * k); }
}

// position of the n-th (0-based) set bit of the 128-bit mask (m0 = tokens 0..63, m1 = 64..127)
__device__ __forceinline__ uint32_t moe_nth_token(uint64_t m0, uint64_t m1, uint32_t n)
{
    const uint32_t c0 = (uint32_t)__popcll(m0);
    uint64_t m = n < c0 ? m0 : m1;
    uint32_t k = n < c0 ? n : n - c0;
    for (; k; --k) m &= m - 1;
    return (uint32_t)__builtin_ctzll(m) + (n < c0 ? 0u : 64u);
}

// A workgroup with fewer messages than waves splits each message into 2, 4 or 8 pieces, one per
// wave, so that a batch of a few tokens is not carried by a single wave while the others idle.
__device__ __forceinline__ uint32_t moe_parts(uint32_t nwaves, uint32_t messages)
{
    uint32_t parts = 1;
    while (messages && parts * 2 * messages <= nwaves) parts *= 2;   // ends: parts doubles, nwaves is fixed
    return parts;
}

// bounded poll of one of the caller's own signals until it is at least `expected`
__device__ __forceinline__ uint64_t moe_poll(const Gin &gin, uint32_t id, uint64_t expected)
{
    uint32_t spins = 0;
    uint64_t v;
    while ((v = gin.read_signal(id)) < expected) {
        if (timed_out(gin.c, spins)) break;
        __builtin_amdgcn_s_sleep(1);
        if (++spins > SPIN_LIMIT) { report(gin.c, DEV_ERR_BARRIER_TIMEOUT, gin.pe); break; }
    }
    return v;
}

// Row g of a PE's flattened list of received rows (local experts in order, within an expert the senders in
// ascending order): which local expert it belongs to, given the experts' first rows ebase[0..epp].
__device__ __forceinline__ uint32_t moe_expert_of_row(const uint32_t *ebase, uint32_t epp, uint32_t g)
{
    uint32_t lo = 0, hi = epp;                  // ebase[lo] <= g < ebase[hi]
    while (hi - lo > 1) {                       // ends: the interval halves
        const uint32_t mid = (lo + hi) >> 1;
        if (ebase[mid] <= g) lo = mid; else hi = mid;
    }
    return lo;
}

// A dispatch count signal carries two numbers: the high half is count + 1, announced once per pair (so that "no
// tokens" differs from "not announced"); the low half grows by the number of messages that have become visible
// -- in one addition for a small batch, in one addition per contributing workgroup for a large one.  The pair
// is complete when the low half has reached the announced count.  Returns the count (0 after a time-out).
__device__ __forceinline__ uint32_t moe_poll_count(const Gin &gin, uint32_t id, bool patient = false, uint32_t nap = 1)
{
    uint32_t spins = 0;
    for (;;) {
        const uint64_t v = gin.read_signal(id);
        const uint32_t hi = (uint32_t)(v >> 32), lo = (uint32_t)v;
        if (hi && lo + 1 == hi) return lo;
        if (timed_out(gin.c, spins)) return 0;
        if (patient) __builtin_amdgcn_s_sleep(100);
        else if (nap > 1) __builtin_amdgcn_s_sleep(16);
        else __builtin_amdgcn_s_sleep(1);
        if (++spins > SPIN_LIMIT) { report(gin.c, DEV_ERR_BARRIER_TIMEOUT, gin.pe); return 0; }
    }
}

// Large batches, receiving side.  The announced count of a pair (high half - 1) is there long before its messages
// are (a sender announces before it sends anything): bounded wait for the announcement alone.
__device__ __forceinline__ uint32_t moe_poll_announced(const Gin &gin, uint32_t id)
{
    uint32_t spins = 0;
    for (;;) {
        const uint32_t hi = (uint32_t)(gin.read_signal(id) >> 32);
        if (hi) return hi - 1;
        if (timed_out(gin.c, spins)) return 0;
        __builtin_amdgcn_s_sleep(8);
        if (++spins > SPIN_LIMIT) { report(gin.c, DEV_ERR_BARRIER_TIMEOUT, gin.pe); return 0; }
    }
}

// Whole wave: returns once all messages of pair `id` are complete (ready[id], in LDS, spares the other waves of
// the workgroup the poll).  No cache maintenance here -- a device-scope acquire is an invalidate of the die's
// whole L2, and one per pair and workgroup (thousands per launch) made the large dispatch 60 % slower.  It is
// not needed either: the workgroup has dropped every stale line once, before its first read of a receive slot
// (the acquire ahead of the packing), and from then on a line of a pair's slots can only enter this die's caches
// through a read, which nobody issues before the pair is complete (slots of different pairs share no line: a
// pair's region is max_tokens messages, a multiple of 128 bytes whenever max_tokens is a multiple of 8, which
// the large-batch path requires).
__device__ __forceinline__ void moe_wait_pair(const Gin &gin, uint32_t id, volatile uint8_t *ready, uint32_t lane)
{
    if (!ready[id]) {
        if (lane == 0) {
            moe_poll_count(gin, id, false, 16);
            ready[id] = 1;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");      // (orders the reads below after the poll)
}

// Sharing N units of work (routes, rows: one message each) among the W workgroups of a PE when the batch is
// large.  The first half goes out in equal fixed ranges, the second in blocks of MOE_BLOCK units that the
// workgroups CLAIM from a counter of the PE -- so a workgroup that the memory serves slowly ends up with fewer
// units and all of them finish within a block or two of each other, while nothing waits for a claim at the
// start.  The eighth wave claims (never more than one range ahead of the range being worked on: a claim ahead
// of need is work nobody else can take over at the end) and publishes ranges through LDS.  Inside the
// workgroup the same idea once more: a message is MOE_PARTS pieces, and waves 0..6 take the workgroup's pieces
// one at a time off a counter in LDS, so that a wave whose pieces come back slowly takes fewer of them.
// work(unit, part) moves one piece.
struct MoeRanges {
    uint32_t rq[MOE_RANGES][2];     // the ranges this workgroup has taken, in order
    uint32_t pub, next;             // ranges published (bit 31: no more will come); pieces handed to waves so far
};

// step(valid, unit, part) is called for every piece a wave takes (valid: there is something to move) and once
// more, with valid = false, when the list has ended.
template <class F>
__device__ __forceinline__ void moe_share_loop(const Ctx &c, MoeRanges &q, uint32_t N, uint32_t W, uint32_t wg, uint64_t *claim,
                                               uint32_t wave, uint32_t lane, F &&step)
{
    // units per claimed block: MOE_BLOCK, or as many as it takes for the lists of the PE's workgroups to hold every
    // block between them (at most N / (2 B) + W + 1 blocks are claimed, a list takes MOE_RANGES - 1 besides the fixed
    // range, and a workgroup whose list is full stops claiming) -- top-k lists of dozens of experts on a team of one
    const uint32_t B = max(MOE_BLOCK, N / (2 * (W * (MOE_RANGES - 3) - 1)) + 1);
    const uint32_t BP = B * MOE_PARTS;                                       // pieces per claimed block
    const uint32_t S = N / (2 * W) / B * B, Ns = S * W;                      // fixed units per workgroup, and in all
    const uint32_t NB = (N - Ns + B - 1) / B;                                // blocks to claim
    const uint32_t k0 = S ? 1u : 0u, p0 = S * MOE_PARTS;                     // ranges, pieces of the fixed part
    if (threadIdx.x == 0) {
        q.rq[0][0] = wg * S; q.rq[0][1] = wg * S + S;
        q.pub = k0; q.next = 0;
    }
    __syncthreads();
    if (wave == MOE_SEND_WAVES) {
        uint32_t k = k0;                                                     // ranges published
        for (;;) {                                                           // ends: the counter only grows
            // wait until the waves have started on the last range published
            for (uint32_t spins = 0; spins < SPIN_LIMIT; ++spins) {
                const uint32_t nx = *(volatile uint32_t *)&q.next;
                const uint32_t at = nx < p0 ? 0u : k0 + (nx - p0) / BP;      // the range piece `nx` belongs to
                if (k <= at + 1) break;
                __builtin_amdgcn_s_sleep(1);
            }
            uint64_t cv = NB;                                                // a full list claims nothing more: the
            if (lane == 0 && k < MOE_RANGES) cv = atomic_fetch_add(claim, 1);   // other workgroups take the rest
            const uint32_t blk = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)min(cv, (uint64_t)0xffffffffu));
            if (blk >= NB) {
                if (lane == 0) *(volatile uint32_t *)&q.pub = k | 0x80000000u;
                break;
            }
            if (lane == 0) {
                *(volatile uint32_t *)&q.rq[k][0] = Ns + blk * B;
                *(volatile uint32_t *)&q.rq[k][1] = min(N, Ns + blk * B + B);
                *(volatile uint32_t *)&q.pub = k + 1;                        // LDS stores of one lane stay in order
            }
            ++k;
        }
    } else if (wave < MOE_SEND_WAVES) {
        for (;;) {
            uint32_t p = 0;
            if (lane == 0) p = __hip_atomic_fetch_add(&q.next, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            p = (uint32_t)__builtin_amdgcn_readfirstlane((int)p);
            const uint32_t k = p < p0 ? 0u : k0 + (p - p0) / BP, within = p < p0 ? p : (p - p0) % BP;
            uint32_t pub, spins = 0;
            while (((pub = *(volatile uint32_t *)&q.pub) & 0x7fffffffu) <= k && !(pub >> 31)) {
                __builtin_amdgcn_s_sleep(1);
                if (++spins > SPIN_LIMIT) { report(c, DEV_ERR_BARRIER_TIMEOUT, blockIdx.x); pub = 0x80000000u; break; }
            }
            if ((pub & 0x7fffffffu) <= k) { step(false, 0u, 0u); break; }    // the list has ended
            const uint32_t unit = *(volatile uint32_t *)&q.rq[k][0] + within / MOE_PARTS;
            step(unit < *(volatile uint32_t *)&q.rq[k][1], unit, within % MOE_PARTS);       // (the last block may be short)
        }
    }
    __syncthreads();
}

template <class F>
__device__ __forceinline__ void moe_share(const Ctx &c, MoeRanges &q, uint32_t N, uint32_t W, uint32_t wg, uint64_t *claim,
                                          uint32_t wave, uint32_t lane, F &&work)
{
    moe_share_loop(c, q, N, W, wg, claim, wave, lane, [&](bool valid, uint32_t unit, uint32_t part) { if (valid) work(unit, part); });
}

// The same sharing with the copies of consecutive pieces overlapped: a wave asks for the vectors of its NEXT piece
// (taking it off the counter, finding its token and its slot, issuing the loads) before it stores the ones it holds,
// so that the loads travel while the stores are issued and the bookkeeping of a piece is not a gap in the wave's
// traffic.  Pieces of up to MOE_PIPE_VECS vectors per lane (both halves of a 14,336-byte token), nothing predicated:
// a lane beyond the end of its piece moves the piece's last vector again.  (Making the wait for the next loads leave
// the stores outstanding as well -- the memory counter of a wave is in order, and a written-through store is only
// acknowledged by memory -- needs stores the compiler can count, i.e. not the `asm` ones; built with raw buffer
// stores carrying the same two coherence bits it measured the same, 90.0 against 89.9 us, and was not kept.)
// prep(unit, part, piece) -> bool issues a piece's loads (false: nothing to move); flush(piece) stores it.
constexpr uint32_t MOE_PIPE_VECS = 7;
struct MoePiece {
    u32x4 v[MOE_PIPE_VECS];
    u32x4 *d;                    // where vector 0 of the piece goes
    uint32_t nv;                 // vectors of the piece (at least 1)
};
struct MoePieceInfo : MoePiece {
    u32x4 info;                  // a message's metadata on its way to the caller's array (first piece only)
    u32x4 *info_d;               // ... or nullptr
};

template <bool CACHED>
__device__ __forceinline__ void moe_piece_load(MoePiece &pc, const u32x4 *__restrict__ s, uint32_t lane)
{
#pragma unroll
    for (uint32_t k = 0; k < MOE_PIPE_VECS; ++k) {
        const u32x4 *at = s + min(lane + 64 * k, pc.nv - 1);
        pc.v[k] = CACHED ? *at : __builtin_nontemporal_load(at);
    }
}

template <bool THROUGH>
__device__ __forceinline__ void moe_piece_store(const MoePiece &pc, uint32_t lane)
{
#pragma unroll
    for (uint32_t k = 0; k < MOE_PIPE_VECS; ++k) {
        u32x4 *at = pc.d + min(lane + 64 * k, pc.nv - 1);
        if (THROUGH) store_through(pc.v[k], at); else __builtin_nontemporal_store(pc.v[k], at);
    }
}

template <class Piece, class FP, class FF>
__device__ __forceinline__ void moe_share_pipe(const Ctx &c, MoeRanges &q, uint32_t N, uint32_t W, uint32_t wg, uint64_t *claim,
                                               uint32_t wave, uint32_t lane, FP &&prep, FF &&flush)
{
    Piece cur, nxt;
    bool have = false;
    moe_share_loop(c, q, N, W, wg, claim, wave, lane, [&](bool valid, uint32_t unit, uint32_t part) {
        if (valid) valid = prep(unit, part, nxt);
        if (have) flush(cur);
        have = valid;
        if (valid) cur = nxt;
    });
}

// After moe_share: the workgroup of the PE that is the last to get here puts the claim counter back to zero
// for the next launch (thread 0 only; `done` counts the workgroups).
__device__ __forceinline__ bool moe_share_done(uint64_t *claim, uint64_t *done, uint32_t W)
{
    if (__hip_atomic_fetch_add(done, 1ull, __ATOMIC_RELAXED, SHMEMX_AGENT) != W - 1) return false;
    __hip_atomic_store(claim, 0ull, __ATOMIC_RELAXED, SHMEMX_AGENT);
    __hip_atomic_store(done, 0ull, __ATOMIC_RELAXED, SHMEMX_AGENT);
    return true;
}

__global__ __launch_bounds__(MOE_THREADS, 4) void k_moe_dispatch(Ctx c, MoeState m, MoeDispatchArgs a)
{
    __shared__ uint64_t mask[MOE_MAX_EXPERTS][2];   // per expert: which of this PE's tokens go there
    __shared__ uint32_t begin[MOE_MAX_EXPERTS + 1]; // small batches: one expert's senders; large: first row of (expert, sender)
    __shared__ uint32_t ebase[MOE_MAX_EXPERTS + 1]; // large batches: first row of every local expert
    __shared__ int16_t s_topk[MOE_MAX_TOKENS * MOE_MAX_TOPK];   // this PE's routing table (expert ids fit 16 bits)
    __shared__ uint32_t rbase[MOE_MAX_EXPERTS + 1]; // large batches: first route of every expert in the PE's flattened list
    __shared__ MoeRanges rq;                        // large batches: the ranges of routes / rows this workgroup takes
    __shared__ uint32_t pbase[MOE_MAX_EXPERTS + 1]; // large batches: first unit of every (sender, local expert) pair in arrival order
    __shared__ uint8_t ready[MOE_MAX_EXPERTS];      // large batches: pair complete and acquired by this workgroup
    __shared__ uint32_t s_last;
    // Workgroup b is number b / npes of PE b mod npes: the chip places workgroup b on die b mod 8, so with 8 PEs all
    // workgroups of a PE share a die and its L2 -- a token is read once per expert it goes to, by different workgroups
    // of its PE, and 128 tokens (1.8 MB) fit one L2 (dispatch of 128 tokens per PE 108.9 -> 104.6 us, 32: 46.5 -> 44.7).
    const uint32_t W = a.wgs_per_pe, P = (uint32_t)c.npes, pe = blockIdx.x % P, wg = blockIdx.x / P;
    const uint32_t E = m.num_experts, T = m.max_tokens, K = m.topk;
    const uint32_t lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const Gin gin{c, m.gin, pe, W};
    const uint32_t ntok = min((uint32_t)max(a.ntok[pe], 0), T);
    const int32_t *topk = a.topk + (size_t)pe * T * K;
    const uint32_t hvecs = (uint32_t)(m.hidden / 16);
    const uint32_t ctl0 = m.epp * P + E;                                     // first control word after the combine flags
    // Large batches are bandwidth-bound and are balanced dynamically; small ones are latency-bound and keep the
    // fixed split, which needs no claim before the first message.  Every workgroup of a PE decides alike.
    const bool bulk = ntok >= MOE_BULK_TOKENS && nwaves > MOE_SEND_WAVES && T % 8 == 0;   // (T % 8: a pair's slots are whole 128-byte lines)

    // ---- routing masks (every workgroup builds its own copy: at most 128 x topk entries) ----
    // The whole table is read, not just the first ntok rows: its loads then do not wait for the load
    // of ntok, and the copy kept in LDS saves the send loop a dependent read per message.
    for (uint32_t i = threadIdx.x; i < 2 * E; i += blockDim.x) (&mask[0][0])[i] = 0;
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < T * K; i += blockDim.x) {
        const int32_t e = topk[i];
        s_topk[i] = (int16_t)(e >= 0 && (uint32_t)e < E ? e : -1);
        if (i >= ntok * K || e < 0) continue;         // beyond the batch, or an unused entry
        const uint32_t t = i / K;
        if ((uint32_t)e >= E) { report(c, DEV_ERR_BAD_TARGET, (uint64_t)pe * T * K + i); continue; }
        const uint64_t bit = 1ull << (t & 63);
        const uint64_t old = __hip_atomic_fetch_or(&mask[e][t >> 6], bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (old & bit) report(c, DEV_ERR_BAD_OP, (uint64_t)pe * T * K + i);   // an expert twice in one token
    }
    __syncthreads();

    // one piece of one message: token number i of expert e (in ascending token order), vectors [part * per, ...)
    auto send_piece = [&](uint32_t e, uint64_t m0, uint64_t m1, uint32_t i, uint32_t part, uint32_t per) {
        const uint32_t owner = e / m.epp, le = e % m.epp;
        const uint32_t t = moe_nth_token(m0, m1, i);
        uint8_t *slot = ptr(c, m.recv_off + (((uint64_t)le * P + pe) * T + i) * m.msg, owner);
        if (part == 0) {
            const uint64_t hit = ballot(lane < K && s_topk[t * K + min(lane, K - 1)] == (int32_t)e);
            const uint32_t j = hit ? (uint32_t)__builtin_ctzll(hit) : 0;
            if (lane == 0) {
                u32x4 meta = {t, pe, j, e};
                store_through(meta, (u32x4 *)slot);
            }
        }
        const uint32_t lo = part * per, cnt = moe_part_vecs(hvecs, lo, per);
        wave_copy16<true, true>((u32x4 *)(slot + MOE_META_BYTES) + lo, (const u32x4 *)(a.x + ((size_t)pe * T + t) * m.hidden) + lo, cnt, lane);
    };

    // large batches: position k of the PE's send order is expert ord(k) (the PE's own experts first, see below)
    const uint32_t erot = (pe * m.epp) % E;
    auto ord = [&](uint32_t k) { const uint32_t e = k + erot; return e >= E ? e - E : e; };
    // ... and what the routes [lo, hi) of this workgroup have made visible is added to their pairs' signals (one
    // lane; a range may span experts, an expert may be split among workgroups)
    auto signal_range = [&](uint32_t lo, uint32_t hi) {
        for (uint32_t k = moe_expert_of_row(rbase, E, lo); lo < hi && k < E; ++k) {
            const uint32_t up = min(hi, rbase[k + 1]);
            if (up <= lo) continue;                                          // an expert without routes
            const uint32_t e = ord(k);
            __hip_atomic_fetch_add(gin.signal_word((e % m.epp) * P + pe, e / m.epp), (uint64_t)(up - lo), __ATOMIC_RELAXED, SHMEMX_AGENT);
            lo = up;
        }
    };
    uint32_t routes = 0;
    if (!bulk) {
        // ---- send: the routes of this workgroup's experts (e = wg mod W), dealt round-robin to its waves ----
        for (uint32_t e = wg; e < E; e += W) routes += (uint32_t)(__popcll(mask[e][0]) + __popcll(mask[e][1]));
        const uint32_t sparts = moe_parts(nwaves, routes), sper = (hvecs + sparts - 1) / sparts;
        uint32_t q = 0;                                                      // running piece number (same in every wave)
        for (uint32_t e = wg; e < E; e += W) {
            const uint64_t m0 = mask[e][0], m1 = mask[e][1];
            const uint32_t n = (uint32_t)(__popcll(m0) + __popcll(m1));
            for (uint32_t i = 0; i < n; ++i)                                 // slot i = i-th token in ascending order
                for (uint32_t part = 0; part < sparts; ++part, ++q)
                    if (q % nwaves == wave) send_piece(e, m0, m1, i, part, sper);
        }
    } else {
        // ---- send, large batch: the PE's routes, flattened in expert order STARTING WITH THE PE'S OWN EXPERTS
        // (position k is expert (k + pe * epp) mod E; route r = token number r - rbase[k] of that expert), shared
        // out by moe_share.  Every PE thus sends to a different owner at any moment, and an owner's messages
        // arrive all through the send phase instead of from everybody at once: the receiving side packs what has
        // arrived while the rest is still on its way (below).
        if (threadIdx.x < 64) {
            const uint32_t per = (E + 63) / 64, k0 = min(lane * per, E), k1 = min(k0 + per, E);
            uint32_t sum = 0;
            for (uint32_t k = k0; k < k1; ++k) { const uint32_t e = ord(k); sum += (uint32_t)(__popcll(mask[e][0]) + __popcll(mask[e][1])); }
            uint32_t incl = sum;
            for (uint32_t d = 1; d < 64; d <<= 1) {                          // inclusive scan over the lanes
                const uint32_t up = (uint32_t)__shfl_up((int)incl, d);
                if (lane >= d) incl += up;
            }
            uint32_t run = incl - sum;
            for (uint32_t k = k0; k < k1; ++k) { const uint32_t e = ord(k); rbase[k] = run; run += (uint32_t)(__popcll(mask[e][0]) + __popcll(mask[e][1])); }
            if (lane == 63) rbase[E] = incl;
        }
        __syncthreads();
        // the announcements (count + 1 in the high half) can go at once: they say nothing about the data
        if (threadIdx.x < 64)
            for (uint32_t k = wg + lane * W; k < E; k += 64 * W) {
                const uint32_t e = ord(k);
                __hip_atomic_fetch_add(gin.signal_word((e % m.epp) * P + pe, e / m.epp), (uint64_t)(rbase[k + 1] - rbase[k] + 1) << 32,
                                       __ATOMIC_RELAXED, SHMEMX_AGENT);
            }
        const uint32_t sper = (hvecs + MOE_PARTS - 1) / MOE_PARTS;
        routes = rbase[E];
        if (sper <= MOE_PIPE_VECS * 64) {
            // (send_piece in two steps: the loads of a piece, and its stores once the next piece's loads are out)
            moe_share_pipe<MoePiece>(c, rq, routes, W, wg, gin.signal_word(ctl0 + MOE_CTL_SEND_CLAIM, pe), wave, lane,
                [&](uint32_t r, uint32_t part, MoePiece &pc) -> bool {
                    const uint32_t k = moe_expert_of_row(rbase, E, r), e = ord(k), i = r - rbase[k];
                    const uint32_t owner = e / m.epp, le = e % m.epp;
                    const uint32_t t = moe_nth_token(mask[e][0], mask[e][1], i);
                    uint8_t *slot = ptr(c, m.recv_off + (((uint64_t)le * P + pe) * T + i) * m.msg, owner);
                    if (part == 0) {
                        const uint64_t hit = ballot(lane < K && s_topk[t * K + min(lane, K - 1)] == (int32_t)e);
                        const uint32_t j = hit ? (uint32_t)__builtin_ctzll(hit) : 0;
                        if (lane == 0) {
                            u32x4 meta = {t, pe, j, e};
                            store_through(meta, (u32x4 *)slot);
                        }
                    }
                    const uint32_t lo = part * sper, cnt = moe_part_vecs(hvecs, lo, sper);
                    if (cnt == 0) return false;
                    pc.d = (u32x4 *)(slot + MOE_META_BYTES) + lo; pc.nv = cnt;
                    moe_piece_load<true>(pc, (const u32x4 *)(a.x + ((size_t)pe * T + t) * m.hidden) + lo, lane);
                    return true;
                },
                [&](const MoePiece &pc) { moe_piece_store<true>(pc, lane); });
        } else {
            moe_share(c, rq, routes, W, wg, gin.signal_word(ctl0 + MOE_CTL_SEND_CLAIM, pe), wave, lane, [&](uint32_t r, uint32_t part) {
                const uint32_t k = moe_expert_of_row(rbase, E, r), e = ord(k);
                send_piece(e, mask[e][0], mask[e][1], r - rbase[k], part, sper);
            });
        }
        // While this workgroup's last stores are on their way (the release below waits for them), it reads ALL the PE's
        // announced counts -- they were sent before any message -- and lays out what it will receive: see the receive
        // phase below.  (Done after the release, these microseconds were a gap between the two phases.)
        {
            const uint32_t npairs = m.epp * P;
            for (uint32_t i = threadIdx.x; i < npairs; i += blockDim.x) {
                const uint32_t n = min(moe_poll_announced(gin, i), T);
                begin[i] = n;
                const uint32_t le = i / P, s = i % P, phase = (pe + P - s) % P;
                pbase[phase * m.epp + le + 1] = n;                           // counts in arrival order, summed up below
                ready[i] = 0;
            }
            __syncthreads();
            for (uint32_t le = threadIdx.x; le < m.epp; le += blockDim.x) {  // counts -> first rows within the expert
                uint32_t run = 0;
                for (uint32_t s = 0; s < P; ++s) {
                    const uint32_t n = begin[le * P + s];
                    begin[le * P + s] = run;
                    run += n;
                }
                ebase[le + 1] = run;
            }
            if (wave == 1) {                                                 // running sum over the pairs: every lane a stretch
                const uint32_t per = (npairs + 63) / 64, q0 = min(lane * per, npairs), q1 = min(q0 + per, npairs);
                uint32_t sum = 0;
                for (uint32_t q = q0; q < q1; ++q) sum += pbase[q + 1];
                uint32_t incl = sum;
                for (uint32_t d = 1; d < 64; d <<= 1) {
                    const uint32_t up = (uint32_t)__shfl_up((int)incl, d);
                    if (lane >= d) incl += up;
                }
                uint32_t run = incl - sum;
                for (uint32_t q = q0; q < q1; ++q) { run += pbase[q + 1]; pbase[q + 1] = run; }
                if (lane == 0) pbase[0] = 0;
            }
            __syncthreads();
            if (threadIdx.x == 0) {
                ebase[0] = 0;
                for (uint32_t le = 0; le < m.epp; ++le) ebase[le + 1] += ebase[le];
            }
            __syncthreads();
            for (uint32_t le = wg; le < m.epp; le += W) {                    // the bookkeeping of an expert: one workgroup
                const uint32_t total = ebase[le + 1] - ebase[le];
                for (uint32_t s = threadIdx.x; s < P; s += blockDim.x) {
                    const uint32_t b = begin[le * P + s], nx = s + 1 < P ? begin[le * P + s + 1] : total;
                    a.recv_range[(((size_t)pe * m.epp + le) * P + s) * 2] = (int32_t)b;
                    a.recv_range[(((size_t)pe * m.epp + le) * P + s) * 2 + 1] = (int32_t)(nx - b);
                }
                if (threadIdx.x == 0) a.recv_count[(size_t)pe * m.epp + le] = (int32_t)total;
            }
        }
    }
    // counts: zero-byte put + SignalAdd per (this PE, expert) pair -- after every wave's messages are
    // complete and one release has made them visible, so a count is never seen before its data
    wg_release();
    if (threadIdx.x < 64) {
        if (routes) quiet();                                                 // nothing was written: nothing to release
        if (!bulk) {
            for (uint32_t e = wg + lane * W; e < E; e += 64 * W) {
                const uint64_t n = (uint64_t)(__popcll(mask[e][0]) + __popcll(mask[e][1]));
                __hip_atomic_fetch_add(gin.signal_word((e % m.epp) * P + pe, e / m.epp), (n + 1) << 32 | n, __ATOMIC_RELAXED, SHMEMX_AGENT);
            }
        } else {
            // what this workgroup sent, range by range
            const uint32_t mine = rq.pub & 0x7fffffffu;
            for (uint32_t k = lane; k < mine; k += 64) signal_range(rq.rq[k][0], rq.rq[k][1]);
            if (lane == 0)
                moe_share_done(gin.signal_word(ctl0 + MOE_CTL_SEND_CLAIM, pe), gin.signal_word(ctl0 + MOE_CTL_SEND_DONE, pe), W);
        }
    }

    if (!bulk) {
        // ---- receive: this workgroup's local experts ----
        for (uint32_t le = wg; le < m.epp; le += W) {
            __syncthreads();                                                 // begin[] of the previous expert is done with
            for (uint32_t s = threadIdx.x; s < P; s += blockDim.x) {
                begin[s + 1] = min(moe_poll_count(gin, le * P + s), T);
                gin.reset_signal(le * P + s);                                // nobody else reads it; next dispatch starts clean
            }
            __syncthreads();
            if (le == wg)            if (threadIdx.x < 64) acquire();                                 // what the signals released is now readable
            wg_acquire();
            if (threadIdx.x == 0) {
                begin[0] = 0;
                for (uint32_t s = 0; s < P; ++s) begin[s + 1] += begin[s];
            }
            __syncthreads();
            const uint32_t total = begin[P];
            const size_t row0 = ((size_t)pe * m.epp + le) * ((size_t)P * T);
            for (uint32_t s = threadIdx.x; s < P; s += blockDim.x) {
                a.recv_range[(((size_t)pe * m.epp + le) * P + s) * 2] = (int32_t)begin[s];
                a.recv_range[(((size_t)pe * m.epp + le) * P + s) * 2 + 1] = (int32_t)(begin[s + 1] - begin[s]);
            }
            if (threadIdx.x == 0) a.recv_count[(size_t)pe * m.epp + le] = (int32_t)total;
            const uint32_t rparts = moe_parts(nwaves, total), rper = (hvecs + rparts - 1) / rparts;
            for (uint32_t u = wave; u < total * rparts; u += nwaves) {
                const uint32_t i = u / rparts, part = u % rparts;
                uint32_t s = 0;
                while (begin[s + 1] <= i) ++s;
                const uint8_t *slot = ptr(c, m.recv_off + (((uint64_t)le * P + s) * T + (i - begin[s])) * m.msg, pe);
                // the metadata is requested before the token and stored after it, so the two reads travel together
                const bool first = part == 0 && lane == 0;
                u32x4 info = {0, 0, 0, 0};
                if (first) info = *(const u32x4 *)slot;
                const uint32_t lo = part * rper, cnt = moe_part_vecs(hvecs, lo, rper);
                wave_copy16<false>((u32x4 *)(a.recv_x + (row0 + i) * m.hidden) + lo, (const u32x4 *)(slot + MOE_META_BYTES) + lo, cnt, lane);
                if (first) *(u32x4 *)(a.recv_info + (row0 + i) * 4) = info;
            }
        }
    } else {
        // ---- receive, large batch: every workgroup of the PE reads ALL the PE's announced counts (they are there
        // long before the messages), and the rows of all local experts are shared out by moe_share (36 experts on
        // 32 workgroups would otherwise leave four workgroups with twice the work) -- in the order in which they
        // ARRIVE: sender s reaches this PE's experts in phase (pe - s) mod P of its send order, so the units are the
        // pairs by phase, then by local expert, and a wave waits only for the pair its own row belongs to.  The
        // workgroups that finish sending early pack what is complete while the last messages are still in flight.
        // The signals are put back to zero by the workgroup of the PE that finishes last.
        const uint32_t npairs = m.epp * P;
        if (threadIdx.x < 64) acquire();                                     // once: see moe_wait_pair
        wg_acquire();
        const uint32_t rper = (hvecs + MOE_PARTS - 1) / MOE_PARTS;
        if (rper <= MOE_PIPE_VECS * 64)
            moe_share_pipe<MoePieceInfo>(c, rq, pbase[npairs], W, wg, gin.signal_word(ctl0 + MOE_CTL_RECV_CLAIM, pe), wave, lane,
                [&](uint32_t g, uint32_t part, MoePieceInfo &pc) -> bool {
                    const uint32_t q = moe_expert_of_row(pbase, npairs, g), i = g - pbase[q];    // pair in arrival order, message of the pair
                    const uint32_t le = q % m.epp, s = (pe + P - q / m.epp) % P;
                    moe_wait_pair(gin, le * P + s, ready, lane);
                    const uint8_t *slot = ptr(c, m.recv_off + (((uint64_t)le * P + s) * T + i) * m.msg, pe);
                    const size_t row = ((size_t)pe * m.epp + le) * ((size_t)P * T) + begin[le * P + s] + i;
                    const uint32_t lo = part * rper, cnt = moe_part_vecs(hvecs, lo, rper);
                    pc.info_d = part == 0 ? (u32x4 *)(a.recv_info + row * 4) : nullptr;
                    pc.info = *(const u32x4 *)slot;                                              // (one request for the wave)
                    if (cnt == 0) { if (pc.info_d && lane == 0) *pc.info_d = pc.info; return false; }
                    pc.d = (u32x4 *)(a.recv_x + row * m.hidden) + lo; pc.nv = cnt;
                    moe_piece_load<false>(pc, (const u32x4 *)(slot + MOE_META_BYTES) + lo, lane);
                    return true;
                },
                [&](const MoePieceInfo &pc) {
                    moe_piece_store<false>(pc, lane);
                    if (pc.info_d && lane == 0) *pc.info_d = pc.info;
                });
        else
        moe_share(c, rq, pbase[npairs], W, wg, gin.signal_word(ctl0 + MOE_CTL_RECV_CLAIM, pe), wave, lane, [&](uint32_t g, uint32_t part) {
            const uint32_t q = moe_expert_of_row(pbase, npairs, g), i = g - pbase[q];        // pair in arrival order, message of the pair
            const uint32_t le = q % m.epp, s = (pe + P - q / m.epp) % P;
            moe_wait_pair(gin, le * P + s, ready, lane);
            const uint8_t *slot = ptr(c, m.recv_off + (((uint64_t)le * P + s) * T + i) * m.msg, pe);
            const size_t row = ((size_t)pe * m.epp + le) * ((size_t)P * T) + begin[le * P + s] + i;
            const bool first = part == 0 && lane == 0;
            u32x4 info = {0, 0, 0, 0};
            if (first) info = *(const u32x4 *)slot;
            const uint32_t lo = part * rper, cnt = moe_part_vecs(hvecs, lo, rper);
            wave_copy16<false>((u32x4 *)(a.recv_x + row * m.hidden) + lo, (const u32x4 *)(slot + MOE_META_BYTES) + lo, cnt, lane);
            if (first) *(u32x4 *)(a.recv_info + row * 4) = info;
        });
        if (threadIdx.x == 0)
            s_last = moe_share_done(gin.signal_word(ctl0 + MOE_CTL_RECV_CLAIM, pe), gin.signal_word(ctl0 + MOE_CTL_RECV_DONE, pe), W);
        __syncthreads();
        if (s_last)                                                          // every workgroup of the PE has read the counts
            for (uint32_t i = threadIdx.x; i < npairs; i += blockDim.x) gin.reset_signal(i);
    }
}

__global__ __launch_bounds__(MOE_THREADS) void k_moe_combine(Ctx c, MoeState m, MoeCombineArgs a)
{
    __shared__ uint32_t begin[MOE_MAX_PES + 1];
    __shared__ uint32_t ebase[MOE_MAX_EXPERTS + 1]; // large batches: first row of every local expert
    __shared__ MoeRanges rq;                        // large batches: the ranges of rows this workgroup returns
    __shared__ int32_t experts[MOE_MAX_TOPK];
    __shared__ uint64_t epoch;   // number of this combine on the object: the flags count combines and are never reset
    const uint32_t W = a.wgs_per_pe, P = (uint32_t)c.npes, pe = blockIdx.x % P, wg = blockIdx.x / P;   // (as in the dispatch)
    const uint32_t T = m.max_tokens, K = m.topk;
    const uint32_t lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const Gin gin{c, m.gin, pe, W};
    const uint32_t flag0 = m.epp * P;                                        // first combine flag ID
    const uint32_t hvecs = (uint32_t)(m.hidden / 16);
    // The count of completed combines lives on the device (a launch replayed from a graph carries no fresh
    // arguments): ctl[0] on every PE, written by the workgroup of the team that was the LAST to read it --
    // every workgroup reads ctl[0] first and only then adds itself to ctl[1] -- at its very end.
    uint64_t *ctl = gin.signal_word(flag0 + m.num_experts + MOE_CTL_COMBINES, pe);
    uint64_t completed = 0, arrival = 0;
    if (threadIdx.x == 0) completed = __hip_atomic_load(ctl, __ATOMIC_RELAXED, SHMEMX_AGENT);   // used after the send phase

    // the row counts of the first expert are requested before the batch size is looked at (two dependent round
    // trips to memory would otherwise open every small combine)
    int32_t n_first = 0;
    if (wg < m.epp && threadIdx.x < P) n_first = a.recv_range[((((size_t)pe * m.epp + wg) * P) + threadIdx.x) * 2 + 1];
    const uint32_t ntok = min((uint32_t)max(a.ntok[pe], 0), T);
    const uint32_t ctl0 = flag0 + m.num_experts;
    const bool bulk = ntok >= MOE_BULK_TOKENS && nwaves > MOE_SEND_WAVES;    // as in the dispatch: large batches are balanced dynamically
    // one piece of one row back to its token's source
    auto return_piece = [&](size_t row, uint32_t part, uint32_t parts, uint32_t per) {
        const u32x4 info = *(const u32x4 *)(a.recv_info + row * 4);          // token, source PE, position, expert
        const uint32_t t = info.x, s = info.y, j = info.z;
        if (t >= T || s >= P || j >= K) { if (lane == 0 && part == 0) report(c, DEV_ERR_BAD_OP, row); return; }
        const uint32_t lo = part * per, cnt = moe_part_vecs(hvecs, lo, per);
        wave_copy16<true>((u32x4 *)ptr(c, m.comb_off + ((uint64_t)t * K + j) * m.hidden, s) + lo,
                    (const u32x4 *)(a.expert_out + row * m.hidden) + lo, cnt, lane);
    };
    if (!bulk) {
        // ---- send: the outputs of this workgroup's local experts go back to the tokens' sources ----
        for (uint32_t le = wg; le < m.epp; le += W) {
            __syncthreads();
            const size_t pair0 = ((size_t)pe * m.epp + le) * P;
            if (threadIdx.x < P) {
                const int32_t n = le == wg ? n_first : a.recv_range[(pair0 + threadIdx.x) * 2 + 1];
                begin[threadIdx.x + 1] = (uint32_t)min(max(n, 0), (int32_t)T);
            }
            __syncthreads();
            if (threadIdx.x == 0) {
                begin[0] = 0;
                for (uint32_t s = 0; s < P; ++s) begin[s + 1] += begin[s];
            }
            __syncthreads();
            const uint32_t total = begin[P];
            const size_t row0 = ((size_t)pe * m.epp + le) * ((size_t)P * T);
            const uint32_t cparts = moe_parts(nwaves, total), cper = (hvecs + cparts - 1) / cparts;
            for (uint32_t u = wave; u < total * cparts; u += nwaves) return_piece(row0 + u / cparts, u % cparts, cparts, cper);
            // flags: zero-byte put + SignalAdd to every destination, after one release for the whole expert
            wg_release();
            if (threadIdx.x < 64) {
                quiet();
                for (uint32_t s = lane; s < P; s += 64)
                    __hip_atomic_fetch_add(gin.signal_word(flag0 + pe * m.epp + le, s), 1ull, __ATOMIC_RELAXED, SHMEMX_AGENT);
            }
        }
    } else {
        // ---- send, large batch: the rows of all local experts, flattened, are shared out by moe_share.  An
        // expert's rows then leave from several workgroups, so its flags can only go once all of them have
        // released: every workgroup counts itself done on a word of the PE after its release, and the last one
        // raises the flags of all the PE's experts (the workgroups finish together: that is what the sharing is for).
        for (uint32_t le = threadIdx.x; le < m.epp; le += blockDim.x) {
            uint32_t run = 0;
            for (uint32_t s = 0; s < P; ++s) run += (uint32_t)min(max(a.recv_range[((((size_t)pe * m.epp + le) * P) + s) * 2 + 1], 0), (int32_t)T);
            ebase[le + 1] = run;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            ebase[0] = 0;
            for (uint32_t le = 0; le < m.epp; ++le) ebase[le + 1] += ebase[le];
        }
        __syncthreads();
        const uint32_t cper = (hvecs + MOE_PARTS - 1) / MOE_PARTS;
        if (cper <= MOE_PIPE_VECS * 64)
            // (return_piece in two steps, see moe_share_pipe)
            moe_share_pipe<MoePiece>(c, rq, ebase[m.epp], W, wg, gin.signal_word(ctl0 + MOE_CTL_COMB_CLAIM, pe), wave, lane,
                [&](uint32_t g, uint32_t part, MoePiece &pc) -> bool {
                    const uint32_t le = moe_expert_of_row(ebase, m.epp, g);
                    const size_t row = ((size_t)pe * m.epp + le) * ((size_t)P * T) + (g - ebase[le]);
                    const u32x4 info = *(const u32x4 *)(a.recv_info + row * 4);      // token, source PE, position, expert
                    const uint32_t t = info.x, s = info.y, j = info.z;
                    if (t >= T || s >= P || j >= K) { if (lane == 0 && part == 0) report(c, DEV_ERR_BAD_OP, row); return false; }
                    const uint32_t lo = part * cper, cnt = moe_part_vecs(hvecs, lo, cper);
                    if (cnt == 0) return false;
                    pc.d = (u32x4 *)ptr(c, m.comb_off + ((uint64_t)t * K + j) * m.hidden, s) + lo; pc.nv = cnt;
                    moe_piece_load<false>(pc, (const u32x4 *)(a.expert_out + row * m.hidden) + lo, lane);
                    return true;
                },
                [&](const MoePiece &pc) { moe_piece_store<true>(pc, lane); });
        else
        moe_share(c, rq, ebase[m.epp], W, wg, gin.signal_word(ctl0 + MOE_CTL_COMB_CLAIM, pe), wave, lane, [&](uint32_t g, uint32_t part) {
            const uint32_t le = moe_expert_of_row(ebase, m.epp, g);
            return_piece(((size_t)pe * m.epp + le) * ((size_t)P * T) + (g - ebase[le]), part, MOE_PARTS, cper);
        });
        wg_release();
        if (threadIdx.x < 64) {
            quiet();
            uint32_t last = 0;
            if (lane == 0) last = moe_share_done(gin.signal_word(ctl0 + MOE_CTL_COMB_CLAIM, pe), gin.signal_word(ctl0 + MOE_CTL_COMB_DONE, pe), W);
            if (__builtin_amdgcn_readfirstlane((int)last))
                for (uint32_t i = lane; i < m.epp * P; i += 64)
                    __hip_atomic_fetch_add(gin.signal_word(flag0 + pe * m.epp + i / P, i % P), 1ull, __ATOMIC_RELAXED, SHMEMX_AGENT);
        }
    }

    if (threadIdx.x == 0) {
        epoch = completed + 1;
        uint64_t one = 1;
        asm volatile("" : "+v"(one) : "v"(completed));   // the arrival is issued only once ctl[0] has been read
        arrival = __hip_atomic_fetch_add(ctl + 1, one, __ATOMIC_RELAXED, SHMEMX_AGENT);   // looked at when the workgroup ends
    }

    // ---- receive: this workgroup's tokens ----
    for (uint32_t t = wg; t < ntok; t += W) {
        __syncthreads();                                                     // also publishes `epoch`
        if (threadIdx.x < K) {
            const int32_t e = a.topk[((size_t)pe * T + t) * K + threadIdx.x];
            const bool ok = e >= 0 && (uint32_t)e < m.num_experts;
            experts[threadIdx.x] = ok ? e : -1;
            if (ok) moe_poll(gin, flag0 + (uint32_t)e, epoch);               // that expert's outputs for this PE are in
        }
        if (threadIdx.x < 64) acquire();
        wg_acquire();
        const u32x4 *slots = (const u32x4 *)ptr(c, m.comb_off + (uint64_t)t * K * m.hidden, pe);
        u32x4 *out = (u32x4 *)(a.combined + ((size_t)pe * T + t) * m.hidden);
        // every slot of the token is loaded, eight at a time, whether or not its route is in use (an
        // unused slot holds old bytes that are not added): loads under a condition would go out one
        // memory round trip after the other
        for (uint32_t v = threadIdx.x; v < hvecs; v += blockDim.x) {
            u32x4 acc = {0, 0, 0, 0};
            for (uint32_t j0 = 0; j0 < K; j0 += 8) {
                u32x4 w[8];
#pragma unroll
                for (uint32_t k = 0; k < 8; ++k) w[k] = __builtin_nontemporal_load(slots + (size_t)min(j0 + k, K - 1) * hvecs + v);
#pragma unroll
                for (uint32_t k = 0; k < 8; ++k)
                    if (j0 + k < K && experts[j0 + k] >= 0) acc += w[k];
            }
            __builtin_nontemporal_store(acc, out + v);
        }
    }
    if (threadIdx.x == 0 && arrival == W - 1) {      // every workgroup of the team has read ctl[0]: this combine is counted
        __hip_atomic_store(ctl + 1, 0ull, __ATOMIC_RELAXED, SHMEMX_AGENT);
        __hip_atomic_store(ctl, completed + 1, __ATOMIC_RELAXED, SHMEMX_AGENT);
    }
}

}  // namespace shmemx

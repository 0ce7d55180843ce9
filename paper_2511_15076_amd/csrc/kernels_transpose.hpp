// Distributed matrix transpose by one-sided gets (an iget-shaped variant of the
// path; the paper has no such operation).  PE p holds rows [p*R, (p+1)*R) of an
// n x n matrix A and produces the same rows of B = A^T.  Row i of B on PE p is
// column p*R + i of A, spread over every PE: as plain igets that is one element
// per 4*n-byte pitch -- a full memory sector per element.  Here a workgroup
// moves a 64 x 64 tile through LDS instead: each tile row is a contiguous get of
// 64 elements from the row's owner, and the transposed tile leaves as 64
// contiguous local stores, so both sides move whole lines.
#pragma once
#include "../../include/mi_shmemx.hpp"

namespace shmemx {

constexpr uint32_t TR_TILE = 64;

struct TransposeArgs {
    uint64_t in_off, out_off;   // symmetric offsets of A's and B's row blocks
    uint64_t n, rows;           // matrix order; rows per PE (n / npes)
    uint32_t wgs_per_pe;
};

template <typename T>
__global__ __launch_bounds__(256) void k_transpose(Ctx c, TransposeArgs a)
{
    __shared__ T tile[TR_TILE][TR_TILE + 1];       // +1: conflict-free column reads
    const uint32_t pe = blockIdx.x / a.wgs_per_pe, wg = blockIdx.x % a.wgs_per_pe;
    constexpr uint32_t WAVES = 4, PER = TR_TILE / WAVES;    // launched with 256 threads: 16 tile rows per thread
    const uint32_t tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const uint64_t tiles_i = (a.rows + TR_TILE - 1) / TR_TILE, tiles_j = (a.n + TR_TILE - 1) / TR_TILE;
    T *out = (T *)ptr(c, a.out_off, pe);
    for (uint64_t t = wg; t < tiles_i * tiles_j; t += a.wgs_per_pe) {
        const uint64_t i0 = (t / tiles_j) * TR_TILE;        // first local output row of the tile
        const uint64_t j0 = (t % tiles_j) * TR_TILE;        // first output column = first source row (global)
        // tile row r = source row j0 + r, columns p*R + i0 .. + 64: a contiguous get from the row's owner;
        // a thread's sixteen gets are all requested before the first one is used
        T v[PER];
#pragma unroll
        for (uint32_t k = 0; k < PER; ++k) {
            const uint64_t j = j0 + ty + k * WAVES, col = i0 + tx;
            v[k] = 0;
            if (j < a.n && col < a.rows) {
                const uint32_t q = (uint32_t)(j / a.rows);
                const T *src = (const T *)ptr(c, a.in_off, q) + (j - (uint64_t)q * a.rows) * a.n + (uint64_t)pe * a.rows + col;
                v[k] = __builtin_nontemporal_load(src);
            }
        }
#pragma unroll
        for (uint32_t k = 0; k < PER; ++k) tile[ty + k * WAVES][tx] = v[k];
        __syncthreads();
#pragma unroll
        for (uint32_t k = 0; k < PER; ++k) {
            const uint32_t r = ty + k * WAVES;
            const uint64_t i = i0 + r, j = j0 + tx;
            if (i < a.rows && j < a.n) __builtin_nontemporal_store(tile[tx][r], out + i * a.n + j);
        }
        __syncthreads();
    }
}

// The same with 16-byte gets and 16-byte stores (four uint32 or two uint64 per lane): a tile row is then
// 16 or 32 lanes wide, so one wave instruction covers four or two tile rows.  Needs rows, i.e. n / npes,
// to be a multiple of the vector length (every vector then lies inside one row block and is 16-byte
// aligned); the host falls back to the element-wise kernel otherwise.  TJ source rows make one tile:
// 64, or 128 for 4-byte elements, which doubles the contiguous run of every output row to 512 bytes
// (runs of 256 bytes reach about 0.65 of the HBM peak in the put / get sweep as well, 512 bytes 0.67).
template <typename T, uint32_t TJ>
__global__ __launch_bounds__(256) void k_transpose_vec(Ctx c, TransposeArgs a)
{
    constexpr uint32_t E = 16 / sizeof(T);                 // elements per vector
    constexpr uint32_t LANES_IN = TR_TILE / E;             // lanes per source row of the tile (64 elements)
    constexpr uint32_t ROWS_IN = 256 / LANES_IN;           // source rows per step of the workgroup
    constexpr uint32_t STEPS_IN = TJ / ROWS_IN;
    constexpr uint32_t LANES_OUT = TJ / E;                 // lanes per output row of the tile (TJ elements)
    constexpr uint32_t ROWS_OUT = 256 / LANES_OUT;
    constexpr uint32_t STEPS_OUT = TR_TILE / ROWS_OUT;
    typedef T vec __attribute__((ext_vector_type(E)));
    __shared__ T tile[TJ][TR_TILE + 1];                    // [source row][local column]; +1: conflict-free column reads
    const uint32_t pe = blockIdx.x / a.wgs_per_pe, wg = blockIdx.x % a.wgs_per_pe;
    const uint32_t vx = threadIdx.x % LANES_IN, ry = threadIdx.x / LANES_IN;
    const uint32_t ox = threadIdx.x % LANES_OUT, oy = threadIdx.x / LANES_OUT;
    const uint64_t tiles_i = (a.rows + TR_TILE - 1) / TR_TILE, tiles_j = (a.n + TJ - 1) / TJ;
    T *out = (T *)ptr(c, a.out_off, pe);
    // Tiles are CLAIMED from a counter of the PE, not dealt (the workgroups of a launch run at unequal speeds, and
    // with equal shares the launch lasts as long as the slowest needs): the first tile of a workgroup is its
    // number, the claim for the next is made when a tile is started and read when it is finished.  The last
    // workgroup of the launch to finish puts the counters back to zero.
    __shared__ uint64_t next_tile;
    uint64_t *const claim = &c.scratch[W_PE_BASE + (uint64_t)pe * W_PE_WORDS + 9];
    const uint64_t ntiles = tiles_i * tiles_j;
    uint64_t got = 0;
    for (uint64_t t = wg; t < ntiles;) {
        if (threadIdx.x == 0) got = atomic_fetch_add_deferred(claim, 1);
        const uint64_t i0 = (t / tiles_j) * TR_TILE, j0 = (t % tiles_j) * TJ;
        vec v[STEPS_IN];
#pragma unroll
        for (uint32_t k = 0; k < STEPS_IN; ++k) {
            const uint64_t j = j0 + ry + k * ROWS_IN, col = i0 + vx * E;   // source row; first local column of the vector
            v[k] = vec(0);
            if (j < a.n && col < a.rows) {                                 // rows % E == 0: a vector is in or out as a whole
                const uint32_t q = (uint32_t)(j / a.rows);
                const T *src = (const T *)ptr(c, a.in_off, q) + (j - (uint64_t)q * a.rows) * a.n + (uint64_t)pe * a.rows + col;
                v[k] = __builtin_nontemporal_load((const vec *)src);
            }
        }
#pragma unroll
        for (uint32_t k = 0; k < STEPS_IN; ++k)
#pragma unroll
            for (uint32_t e = 0; e < E; ++e) tile[ry + k * ROWS_IN][vx * E + e] = v[k][e];
        __syncthreads();
#pragma unroll
        for (uint32_t k = 0; k < STEPS_OUT; ++k) {
            const uint32_t r = oy + k * ROWS_OUT;                          // tile column = local output row
            const uint64_t i = i0 + r, j = j0 + ox * E;
            if (i < a.rows && j < a.n) {                                   // n % E == 0 as well
                vec o;
#pragma unroll
                for (uint32_t e = 0; e < E; ++e) o[e] = tile[ox * E + e][r];
                __builtin_nontemporal_store(o, (vec *)(out + i * a.n + j));
            }
        }
        if (threadIdx.x == 0) next_tile = (uint64_t)a.wgs_per_pe + got;
        __syncthreads();
        t = next_tile;
    }
    if (threadIdx.x == 0) {
        // (a workgroup that never entered the loop has made no claim; every other one has read its last)
        uint64_t *const done = &c.scratch[W_WORK + 9];
        if (atomic_fetch_add(done, 1) == (uint64_t)gridDim.x - 1) {
            for (uint32_t p = 0; p < (uint32_t)c.npes; ++p)
                __hip_atomic_store(&c.scratch[W_PE_BASE + (uint64_t)p * W_PE_WORDS + 9], 0ull, __ATOMIC_RELAXED, SHMEMX_AGENT);
            __hip_atomic_store(done, 0ull, __ATOMIC_RELAXED, SHMEMX_AGENT);
        }
    }
}

}  // namespace shmemx

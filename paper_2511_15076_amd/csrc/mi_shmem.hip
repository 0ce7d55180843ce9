// mi_shmem: host side of the C ABI declared in include/mi_shmem.h plus the
// gfx950 kernels it launches.  One translation unit; the kernels live in the
// headers included below and are built from the primitives in include/mi_shmemx.hpp.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <thread>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>
#include <rocprim/device/device_segmented_radix_sort.hpp>   // once per graph: shmem_bfs_create sorts the rows of its adjacency

#include "../../include/mi_shmem.h"
#include "host_logic.hpp"
#include "../../include/mi_shmemx.hpp"
#include "kernels_copy.hpp"
#include "kernels_stream.hpp"
#include "kernels_amo.hpp"
#include "kernels_hash.hpp"
#include "kernels_bfs.hpp"
#include "kernels_sync.hpp"
#include "kernels_moe.hpp"
#include "proxy.hpp"
#include "kernels_transpose.hpp"

namespace {

constexpr size_t GRAN = hostlogic::GRAN;   // allocator granularity / minimum alignment
constexpr int WG_THREADS = 256;    // 4 wavefronts per workgroup
constexpr int HASH_LOOKUP_KIF = 4;  // keys in flight per lane quad in the sector-wide lookup
constexpr uint32_t BFS_ALPHA = 30, BFS_BETA = 24;  // default direction thresholds (measured best on R-MAT scale 24)
constexpr uint32_t BFS_SORT_DIV = 64;              // frontiers from nverts / 64 vertices on are expanded in vertex order

struct Host {
    bool init = false;
    int npes = 0;
    size_t seg = 0;
    uint8_t *heap = nullptr;
    uint64_t *scratch = nullptr;
    hipStream_t stream = nullptr;
    int num_cus = 0;
    int wall_khz = 100000;         // rate of the constant-rate clock the streaming copy paces itself by
    bool stream_dynamic = true;    // bandwidth cells claim their tasks dynamically (kernels_stream.hpp)
    int bfs_sort_rows = 1;         // BFS: the rows of the library's adjacency are sorted by the neighbours' degree rank
    uint32_t bfs_sort_div = 0;     // BFS: frontiers of nverts / this many vertices and more are expanded in vertex order (0: never)
    double stream_pace_ns = 0;     // pacing of the streaming copy: ns per 4 KiB task and workgroup when 256 workgroups stream
    bool cooperative = false;      // cooperative launches for kernels with in-kernel waits
    hostlogic::SymAllocator alloc; // symmetric offsets (guarded by mu)
    uint64_t *pinned = nullptr;    // small host staging area (error word, BFS counts)
    std::mutex mu;
    std::vector<struct shmem_proxy *> proxies;   // live proxy objects (their threads are stopped at finalize)
    // live objects that own synchronisation words in the heap (signal arrays, team barrier words): after a
    // barrier time-out their words are half-advanced and are cleared together with the scratch words
    std::vector<shmemx::GinState> sync_words;
} H;

struct BfsGraph {
    shmemx::BfsState st;
    int wgs_per_pe;
    int mode;          // SHMEM_BFS_TOP_DOWN / DIRECTION_OPTIMIZING / BOTTOM_UP
    bool canonical;    // rewrite the parents into the canonical tree after the search
    uint32_t alpha, beta;  // direction thresholds
    uint64_t nnz;      // CSR entries (sum of all row lengths)
    uint32_t n_long;   // vertices with rows of BIG_DEGREE entries and more: the first n_long of the degree ranking
    void *allocs[12];
    int nallocs;
    // the graph in the library's numbering (device memory the library allocates at creation and frees at destruction)
    uint32_t nverts_orig;
    uint64_t *d_row_int;
    uint32_t *d_nbr_int, *d_to_int, *d_to_orig;
    std::vector<uint32_t> to_int;    // host copy: where the root of a search lives
    // the last search, level by level (host clock around each level's launches and its hand-over; the first 64)
    uint32_t last_levels;
    float last_level_us[64];
    uint8_t last_level_bottom_up[64];
};

inline shmemx::Ctx ctx() { return shmemx::Ctx{H.heap, (uint64_t)H.seg, H.scratch, H.npes}; }
inline bool pe_ok(int pe) { return pe >= 0 && pe < H.npes; }

// symmetric address -> offset in unsigned arithmetic: an address below the heap wraps to a huge offset and
// a null pointer maps to the largest one, so both fail the range checks
inline uint64_t off_of(const void *sym)
{
    return sym ? (uint64_t)((uintptr_t)sym - (uintptr_t)H.heap) : UINT64_MAX;
}

// symmetric address -> offset; checks [off, off+span) lies inside a segment
inline int sym_off(const void *sym, uint64_t span, uint64_t *off)
{
    const uint64_t o = off_of(sym);
    if (!hostlogic::range_in(H.seg, o, span)) return SHMEM_ERR_OUT_OF_RANGE;
    *off = o;
    return SHMEM_OK;
}

using hostlogic::strided_span;

// npes * wgs_per_pe workgroups must be a sane grid (the product is formed in 64 bits)
constexpr uint64_t MAX_GRID = 1u << 22;
inline bool grid_fits(int wgs_per_pe) { return wgs_per_pe >= 1 && (uint64_t)H.npes * (uint64_t)wgs_per_pe <= MAX_GRID; }

inline int hip_rc(hipError_t e) { return e == hipSuccess ? SHMEM_OK : SHMEM_ERR_DEVICE; }
inline int launched() { return hip_rc(hipGetLastError()); }

// A stand-alone put / get: large copies with 16-byte aligned ends stream through the pipelined loop on
// two workgroups per CU (the shape that measured best for one stream), everything else takes the
// generic wave copy.
int launch_copy(uint8_t *dst, const uint8_t *src, size_t n);

// workgroups for a stand-alone copy of n bytes: 16 KiB per workgroup, capped at 8 per CU
inline int wgs_for_bytes(size_t n)
{
    size_t w = (n + 16383) / 16384;
    size_t cap = (size_t)std::max(1, H.num_cus) * 8;
    return (int)std::max<size_t>(1, std::min(w, cap));
}

// Pacing of the streaming copy (kernels_stream.hpp) for a launch of nwg workgroups, in 1/256 ticks of the
// constant-rate clock per task and workgroup.  The target is a chip-wide task rate: 256 workgroups issue one
// 4 KiB task each per STREAM_PACE_NS, i.e. 3.33 TB/s of reads and as much of writes, a few per cent under
// what the memory system sustains for a copy (about 6.8 TB/s of traffic; beyond that it congests and
// delivers 5.5).  Fewer workgroups get proportionally shorter periods (a single compute unit cannot
// reach them, so small launches run unpaced in effect).
constexpr double STREAM_PACE_NS = 315.0;
uint32_t stream_period(unsigned nwg)
{
    const double ns = H.stream_pace_ns * (double)nwg / 256.0;
    const double ticks = ns * (double)H.wall_khz / 1e6;
    return (uint32_t)(ticks * 256.0 + 0.5);
}

int launch_copy(uint8_t *dst, const uint8_t *src, size_t n)
{
    const bool aligned = (((uintptr_t)dst | (uintptr_t)src) & 15) == 0;
    if (n >= (32u << 20) && aligned && n / shmemx::ST_CHUNK < UINT32_MAX) {
        // whole 4 KiB tasks through the wave-specialised streaming copy, one workgroup per compute unit;
        // what is left (under 4 KiB) through the generic copy
        const uint32_t chunks = (uint32_t)(n / shmemx::ST_CHUNK);
        const unsigned grid = (unsigned)std::max(1, H.num_cus);
        hipLaunchKernelGGL(shmemx::k_copy_stream_lds, dim3(grid), dim3(shmemx::ST_THREADS), 0, H.stream, dst, src, chunks,
                           stream_period(grid));
        const size_t done = (size_t)chunks * shmemx::ST_CHUNK;
        if (n > done) hipLaunchKernelGGL(shmemx::k_copy, dim3(1), dim3(WG_THREADS), 0, H.stream, dst + done, src + done, n - done);
    } else if (n >= (1u << 20) && aligned) {
        const size_t want = (n + 16383) / 16384;
        const size_t grid = std::min<size_t>(want, (size_t)std::max(1, H.num_cus) * 2);
        hipLaunchKernelGGL(shmemx::k_copy_stream, dim3((unsigned)grid), dim3(WG_THREADS), 0, H.stream, dst, src, n);
    } else {
        hipLaunchKernelGGL(shmemx::k_copy, dim3(wgs_for_bytes(n)), dim3(WG_THREADS), 0, H.stream, dst, src, n);
    }
    return launched();
}

// co-residency limit for kernels that contain an in-kernel barrier
template <typename K>
int max_resident_wgs(K kernel, int threads = WG_THREADS)
{
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0) != hipSuccess) return 0;
    // gfx950 hands out its 160 KiB of LDS per compute unit in units of 320 dwords; the runtime's figure has been
    // seen to count a workgroup's LDS as it stands (three workgroups of 54,352 bytes, which round up to 55,040
    // each and do not fit: the launch ended in its bounded waits), and a launch that is let through on it waits
    // for workgroups that never start
    hipFuncAttributes fa;
    if (hipFuncGetAttributes(&fa, (const void *)kernel) != hipSuccess) return 0;
    if (fa.sharedSizeBytes > 0) {
        constexpr size_t LDS_PER_CU = 160 * 1024, LDS_UNIT = 1280;
        const size_t need = (fa.sharedSizeBytes + LDS_UNIT - 1) / LDS_UNIT * LDS_UNIT;
        per_cu = (int)std::min<size_t>((size_t)per_cu, LDS_PER_CU / need);
    }
    return per_cu * H.num_cus;
}

void proxy_stop_and_free(struct shmem_proxy *p);   // defined with the proxy executor below

// End of a BFS level: one launch builds the next frontier's bitmap and degree sum (direction-optimising
// modes), and its last workgroup sums the frontier size, resets the per-level counters and writes the
// level counters plus a fresh sequence number into the pinned page.  The host spins on the sequence word
// (no copy, no stream synchronisation), looking at the stream every so often so that a failed launch
// cannot make it wait for ever.
int bfs_level_end(const shmemx::BfsState &s, uint32_t next, bool do_front, bool do_degree, int wgs_per_pe,
                  uint64_t *counts)
{
    static uint64_t seq = 0;
    ++seq;
    // the frontier bitmap alone is a pass over 1/8 byte per vertex: a few workgroups per PE (fewer arrivals to count)
    const unsigned grid = (unsigned)H.npes * (unsigned)(do_degree ? wgs_per_pe : do_front ? std::min(wgs_per_pe, 8) : 1);
    hipLaunchKernelGGL(shmemx::k_bfs_level_end, dim3(grid), dim3(WG_THREADS), 0, H.stream, ctx(), s, next,
                       (int)do_front, (int)do_degree, counts, seq);
    if (int rc = launched()) return rc;
    const auto t0 = std::chrono::steady_clock::now();
    for (uint32_t spins = 0; __atomic_load_n(counts + 3, __ATOMIC_ACQUIRE) != seq; ++spins) {
        if ((spins & 0xFFFF) == 0xFFFF) {
            const hipError_t q = hipStreamQuery(H.stream);
            if (q != hipSuccess && q != hipErrorNotReady) return SHMEM_ERR_DEVICE;
            if (q == hipSuccess && __atomic_load_n(counts + 3, __ATOMIC_ACQUIRE) != seq) return SHMEM_ERR_DEVICE;
            if (std::chrono::steady_clock::now() - t0 > std::chrono::seconds(30)) return SHMEM_ERR_DEVICE;
        }
    }
    return SHMEM_OK;
}

// Launch of a kernel whose workgroups wait for one another (in-kernel barriers, signals): the callers
// have checked that the whole grid fits the device at once (max_resident_wgs), the stream runs one
// kernel at a time, and every in-kernel wait is bounded.  An ordinary launch is used by default: a
// cooperative launch gives the same residency as a formal guarantee but measured about 16 us more per
// launch here, which is most of a small dispatch.  MI_SHMEM_COOPERATIVE_LAUNCH=1 selects it.
int launch_resident(const void *kernel, dim3 grid, dim3 block, void **args)
{
    if (H.cooperative) return hip_rc(hipLaunchCooperativeKernel(kernel, grid, block, args, 0, H.stream));
    return hip_rc(hipLaunchKernel(kernel, grid, block, args, 0, H.stream));
}

void sync_words_add(const shmemx::GinState &g)
{
    std::lock_guard<std::mutex> lk(H.mu);
    H.sync_words.push_back(g);
}
void sync_words_remove(const shmemx::GinState &g)
{
    std::lock_guard<std::mutex> lk(H.mu);
    for (size_t i = 0; i < H.sync_words.size(); ++i)
        if (H.sync_words[i].signals_off == g.signals_off && H.sync_words[i].counters_off == g.counters_off) {
            H.sync_words.erase(H.sync_words.begin() + (long)i);
            return;
        }
}

// ---------------------------------------------------------------------------
// Scratch words that live in the code object, for shmem_op_batch_noalloc: callers that cannot allocate (code
// under graph capture, serving loops, harnesses that forbid it) get the executor's barrier and fault words from
// here instead of from a buffer of their own.  Each GPU that loads the library holds its own copy of the array
// until the process ends.  In host code the array's name is only a stand-in: the device address is looked up
// once per device (with that device current) and kept; kernels, fills and copies get that pointer.
constexpr int NOALLOC_MAX_PES = 64;
constexpr size_t NOALLOC_WORDS = shmemx::W_PE_BASE + (size_t)NOALLOC_MAX_PES * shmemx::W_PE_WORDS;   // 4160 words = 33,280 bytes
constexpr int NOALLOC_MAX_DEVICES = 64;
static __device__ __align__(256) uint64_t scratch[NOALLOC_WORDS];

struct NoallocDevice {
    uint64_t *ptr = nullptr;       // device address of this device's copy of `scratch`
    int num_cus = 0;
    int resident_small = 0, resident_stream = 0;   // co-residency limits of the two executor instances
    bool ready = false;
};
NoallocDevice noalloc_dev[NOALLOC_MAX_DEVICES];
std::mutex noalloc_mu;

__global__ void k_fill_zero(uint64_t *p, uint32_t n)
{
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = 0;
}
__global__ void k_fault_out(const uint64_t *words, uint64_t *out)
{
    if (threadIdx.x < 2) out[threadIdx.x] = __hip_atomic_load(&words[threadIdx.x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Set-up for the current device, on the first call there.
int noalloc_setup(NoallocDevice **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return SHMEM_ERR_DEVICE;
    if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) return SHMEM_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> g(noalloc_mu);
    NoallocDevice &d = noalloc_dev[dev];
    if (!d.ready) {
        uint64_t *ptr = nullptr;
        if (hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SHMEM_ERR_DEVICE;
        int cus = 0, per_cu_small = 0, per_cu_stream = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) return SHMEM_ERR_DEVICE;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_small, shmemx::k_op_batch<false>, WG_THREADS, 0) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_stream, shmemx::k_op_batch<true>, WG_THREADS, 0) != hipSuccess)
            return SHMEM_ERR_DEVICE;
        d.ptr = ptr; d.num_cus = cus; d.resident_small = per_cu_small * cus; d.resident_stream = per_cu_stream * cus;
        d.ready = true;
    }
    *out = &d;
    return SHMEM_OK;
}

// Bandwidth cells -- contiguous messages of whole 4 KiB tasks with 16-byte aligned placement, asked for with at
// least one workgroup per compute unit and enough tasks to fill the rings -- go through the streaming copy: one
// wave-specialised workgroup per compute unit, team = compute units / PEs.  Returns that team size, or 0 for
// the cells that stay on the register-pipelined kernel.
// How a sweep cell is launched.  1: streaming copy with dynamic claiming of 4 KiB tasks (whole multiples of 4 KiB,
// whole blocks of tasks, enough blocks that the fixed first blocks of every workgroup are a small part);
// 3: streaming copy with dynamic claiming of 1 KiB rows (any 16-byte multiple from 1 KiB up whose last row wastes
// less than a tenth of the message's turns); 2: streaming copy with fixed shares (whole 4 KiB tasks, at least a
// ring's worth per workgroup); 0: the register-pipelined kernel.  All streaming launches need 16-byte aligned
// placement and at least one workgroup per compute unit asked for.  *team_out: workgroups per PE of the streaming
// launch (compute units / PEs).
int sweep_stream_kind(bool is_strided, uint64_t count, uint64_t remote_slot, uint64_t local_slot, uint64_t roff,
                      uint64_t loff, uint64_t nslots, int ops_per_pe, int wgs_per_pe, uint32_t *team_out)
{
    if (is_strided || count == 0) return 0;
    if ((count | remote_slot | local_slot | roff | loff) & 15) return 0;
    const uint32_t team = (uint32_t)(H.num_cus / H.npes);
    if (team < 1 || (uint64_t)H.npes * (uint64_t)wgs_per_pe < (uint64_t)H.num_cus || nslots > UINT32_MAX) return 0;
    *team_out = team;
    const bool whole = count % shmemx::ST_CHUNK == 0;
    const uint64_t ntasks = (count / shmemx::ST_CHUNK) * (uint64_t)ops_per_pe;
    const bool dynamic = H.stream_dynamic && team > 1;
    if (whole && dynamic && ntasks % shmemx::ST_BLOCK == 0 && ntasks < (1ull << 31) &&
        ntasks / shmemx::ST_BLOCK >= 2ull * shmemx::ST_STATIC * team) return 1;
    const uint64_t rows_per_block = 4 * shmemx::ST_BLOCK;
    if (dynamic && (count == 512 || (count == 256 && wgs_per_pe < 128))) {
        // several messages to a row: whole groups only, a group never wraps round the slots.  (Measured at 65,536
        // messages per PE, launches of 30 to 90 us in which the streaming kernel's start and end weigh: 512 bytes
        // 0.65 / 0.70 / 0.73 of peak on the register path with 32 / 64 / 256 workgroups per PE asked for, 0.75 here;
        // 256 bytes 0.60 / 0.67 / 0.70 against 0.68; 128 bytes 0.57 / 0.58 / 0.62 against 0.55, so those stay.)
        const uint64_t per_row = 1024 / count;
        if (ops_per_pe % per_row == 0 && nslots % per_row == 0 && std::max(remote_slot, local_slot) * per_row < (1ull << 32) &&
            (uint64_t)ops_per_pe / per_row / rows_per_block >= 2ull * shmemx::ST_STATIC * team) return 4;
        return 0;
    }
    const uint64_t rpo = (count + 1023) / 1024, nrows = rpo * (uint64_t)ops_per_pe;
    if (dynamic && count * 10 >= rpo * 1024 * 9 && nrows < (1ull << 31) &&
        nrows / rows_per_block >= 2ull * shmemx::ST_STATIC * team) return 3;
    if (!whole || ntasks >= UINT32_MAX || ntasks < (uint64_t)team * shmemx::ST_RING) return 0;
    return 2;
}

}  // namespace

extern "C" {

const char *shmem_strerror(int status)
{
    switch (status) {
    case SHMEM_OK: return "ok";
    case SHMEM_ERR_NOT_INIT: return "library not initialised";
    case SHMEM_ERR_ALREADY_INIT: return "library already initialised";
    case SHMEM_ERR_INVALID_ARG: return "invalid argument";
    case SHMEM_ERR_INVALID_PE: return "PE out of range";
    case SHMEM_ERR_OUT_OF_RANGE: return "address or range outside the symmetric segment";
    case SHMEM_ERR_ALIGN: return "misaligned address or size";
    case SHMEM_ERR_NOMEM: return "symmetric heap exhausted";
    case SHMEM_ERR_BAD_FREE: return "not an address returned by shmem_malloc / shmem_align";
    case SHMEM_ERR_DEVICE: return "a HIP runtime call failed";
    case SHMEM_ERR_DEVICE_FAULT: return "an operation was rejected on the device";
    default: return "unknown status";
    }
}

size_t shmem_scratch_bytes(int npes)
{
    if (npes < 1) return 0;
    size_t words = shmemx::W_PE_BASE + (size_t)npes * shmemx::W_PE_WORDS;
    return (words * 8 + 255) / 256 * 256;
}

// False only when the runtime knows the allocation that holds p and it ends before p + bytes.  (A
// pointer the runtime cannot describe is left to the first runtime call that uses it.)
static bool device_range_too_small(const void *p, size_t bytes)
{
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    if (hipMemGetAddressRange(&base, &size, (hipDeviceptr_t)p) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return (uintptr_t)p + bytes > (uintptr_t)base + size;
}

int shmem_init(int npes, size_t heap_bytes_per_pe, void *dev_heap, void *dev_scratch, void *hip_stream)
{
    std::lock_guard<std::mutex> g(H.mu);
    if (H.init) return SHMEM_ERR_ALREADY_INIT;
    if (npes < 1 || npes > 65536 || heap_bytes_per_pe == 0 || !dev_heap || !dev_scratch) return SHMEM_ERR_INVALID_ARG;
    if (heap_bytes_per_pe % GRAN || (uintptr_t)dev_heap % GRAN || (uintptr_t)dev_scratch % GRAN) return SHMEM_ERR_ALIGN;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return SHMEM_ERR_DEVICE;
    if (heap_bytes_per_pe > SIZE_MAX / (size_t)npes) return SHMEM_ERR_INVALID_ARG;
    if (device_range_too_small(dev_heap, (size_t)npes * heap_bytes_per_pe) ||
        device_range_too_small(dev_scratch, shmem_scratch_bytes(npes))) return SHMEM_ERR_OUT_OF_RANGE;
    hipStream_t s = (hipStream_t)hip_stream;
    if (hipMemsetAsync(dev_scratch, 0, shmem_scratch_bytes(npes), s) != hipSuccess) return SHMEM_ERR_DEVICE;
    if (hipStreamSynchronize(s) != hipSuccess) return SHMEM_ERR_DEVICE;
    uint64_t *pinned = nullptr;
    if (hipHostMalloc((void **)&pinned, 4096, hipHostMallocMapped | hipHostMallocCoherent) != hipSuccess) return SHMEM_ERR_DEVICE;
    memset(pinned, 0, 4096);
    H.npes = npes; H.seg = heap_bytes_per_pe; H.heap = (uint8_t *)dev_heap; H.scratch = (uint64_t *)dev_scratch;
    H.stream = s; H.num_cus = prop.multiProcessorCount; H.pinned = pinned;
    const char *coop = getenv("MI_SHMEM_COOPERATIVE_LAUNCH");
    H.cooperative = coop && coop[0] == '1';
    int khz = 0;
    H.wall_khz = (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) == hipSuccess && khz > 0) ? khz : 100000;
    (void)hipGetLastError();
    const char *pace = getenv("MI_SHMEM_STREAM_PACE_NS");     // measurement aid: 0 = unpaced
    H.stream_pace_ns = pace ? atof(pace) : STREAM_PACE_NS;
    if (!(H.stream_pace_ns >= 0.0 && H.stream_pace_ns < 1e6)) H.stream_pace_ns = STREAM_PACE_NS;
    const char *sortdiv = getenv("MI_SHMEM_BFS_SORT_DIV");    // measurement aid: 0 = frontiers are never put in vertex order
    H.bfs_sort_div = sortdiv ? (uint32_t)strtoul(sortdiv, nullptr, 10) : BFS_SORT_DIV;
    const char *sortrows = getenv("MI_SHMEM_BFS_SORT_ROWS");            // measurement aid: 0 = rows left in four classes of rank
    H.bfs_sort_rows = sortrows ? atoi(sortrows) != 0 : 1;
    const char *dyn = getenv("MI_SHMEM_STREAM_DYNAMIC");
    H.stream_dynamic = !dyn || atoi(dyn) != 0;
    H.alloc.reset((uint64_t)(uintptr_t)dev_heap, (uint64_t)heap_bytes_per_pe);
    H.init = true;
    return SHMEM_OK;
}

int shmem_finalize(void)
{
    std::lock_guard<std::mutex> g(H.mu);
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    hipError_t e = hipStreamSynchronize(H.stream);
    while (!H.proxies.empty()) proxy_stop_and_free(H.proxies.back());   // no thread outlives the heap it serves
    if (H.pinned) (void)hipHostFree(H.pinned);
    H.pinned = nullptr; H.init = false; H.npes = 0; H.heap = nullptr; H.scratch = nullptr;
    H.alloc.clear();
    H.sync_words.clear();
    return hip_rc(e);
}

int shmem_n_pes(void) { return H.init ? H.npes : 0; }

void *shmem_align(size_t alignment, size_t nbytes)
{
    std::lock_guard<std::mutex> g(H.mu);
    if (!H.init) return nullptr;
    const uint64_t off = H.alloc.align(alignment, nbytes);
    return off == UINT64_MAX ? nullptr : H.heap + off;
}

void *shmem_malloc(size_t nbytes) { return shmem_align(GRAN, nbytes); }

int shmem_free(void *sym)
{
    std::lock_guard<std::mutex> g(H.mu);
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    const uint8_t *p = (const uint8_t *)sym;
    if (!p || p < H.heap || p >= H.heap + H.seg) return SHMEM_ERR_BAD_FREE;
    return H.alloc.release((uint64_t)(p - H.heap)) ? SHMEM_OK : SHMEM_ERR_BAD_FREE;
}

void *shmem_ptr(const void *sym, int pe)
{
    if (!H.init || !pe_ok(pe)) return nullptr;
    const uint8_t *p = (const uint8_t *)sym;
    if (!p || p < H.heap || p >= H.heap + H.seg) return nullptr;
    return (void *)(p + (size_t)pe * H.seg);
}

// ---------------------------------------------------------------------------
int shmem_put(int pe_self, void *dst_sym, const void *src_local, size_t nbytes, int pe)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    const uint64_t off = off_of(dst_sym);
    if (int rc = hostlogic::check_contig(H.npes, H.seg, pe_self, pe, off, nbytes)) return rc;
    if (nbytes == 0) return SHMEM_OK;
    if (!src_local) return SHMEM_ERR_INVALID_ARG;
    uint8_t *dst = H.heap + (size_t)pe * H.seg + off;
    return launch_copy(dst, (const uint8_t *)src_local, nbytes);
}

int shmem_get(int pe_self, void *dst_local, const void *src_sym, size_t nbytes, int pe)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    const uint64_t off = off_of(src_sym);
    if (int rc = hostlogic::check_contig(H.npes, H.seg, pe_self, pe, off, nbytes)) return rc;
    if (nbytes == 0) return SHMEM_OK;
    if (!dst_local) return SHMEM_ERR_INVALID_ARG;
    const uint8_t *src = H.heap + (size_t)pe * H.seg + off;
    return launch_copy((uint8_t *)dst_local, src, nbytes);
}

static int strided_common(int pe_self, const void *sym, const void *local, ptrdiff_t sym_stride,
                          ptrdiff_t local_stride, size_t nelems, size_t eb, int pe, uint64_t *off)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    *off = off_of(sym);
    if (int rc = hostlogic::check_strided(H.npes, H.seg, pe_self, pe, *off, sym_stride, (uint64_t)(uintptr_t)local,
                                          local_stride, nelems, eb)) return rc;
    if (nelems && !local) return SHMEM_ERR_INVALID_ARG;
    return SHMEM_OK;
}

int shmem_iput(int pe_self, void *dst_sym, const void *src_local, ptrdiff_t dst_stride, ptrdiff_t src_stride,
               size_t nelems, size_t elem_bytes, int pe)
{
    uint64_t off;
    if (int rc = strided_common(pe_self, dst_sym, src_local, dst_stride, src_stride, nelems, elem_bytes, pe, &off)) return rc;
    if (nelems == 0) return SHMEM_OK;
    uint8_t *dst = H.heap + (size_t)pe * H.seg + off;
    hipLaunchKernelGGL(shmemx::k_strided, dim3(wgs_for_bytes(nelems * 16)), dim3(WG_THREADS), 0, H.stream, dst,
                       (const uint8_t *)src_local, (int64_t)dst_stride, (int64_t)src_stride, nelems,
                       (uint32_t)elem_bytes);
    return launched();
}

int shmem_iget(int pe_self, void *dst_local, const void *src_sym, ptrdiff_t dst_stride, ptrdiff_t src_stride,
               size_t nelems, size_t elem_bytes, int pe)
{
    uint64_t off;
    if (int rc = strided_common(pe_self, src_sym, dst_local, src_stride, dst_stride, nelems, elem_bytes, pe, &off)) return rc;
    if (nelems == 0) return SHMEM_OK;
    const uint8_t *src = H.heap + (size_t)pe * H.seg + off;
    hipLaunchKernelGGL(shmemx::k_strided, dim3(wgs_for_bytes(nelems * 16)), dim3(WG_THREADS), 0, H.stream,
                       (uint8_t *)dst_local, src, (int64_t)dst_stride, (int64_t)src_stride, nelems,
                       (uint32_t)elem_bytes);
    return launched();
}

static int amo_single(int kind, int pe_self, uint64_t *sym, uint64_t a, uint64_t b, int pe, uint64_t *dev_result)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    const uint64_t off = off_of(sym);
    if (int rc = hostlogic::check_amo(H.npes, H.seg, pe_self, pe, off)) return rc;
    if ((uintptr_t)dev_result % 8) return SHMEM_ERR_ALIGN;
    uint64_t *target = (uint64_t *)(H.heap + (size_t)pe * H.seg + off);
    hipLaunchKernelGGL(shmemx::k_amo_single, dim3(1), dim3(64), 0, H.stream, kind, target, a, b, dev_result);
    return launched();
}

int shmem_put_signal(int pe_self, void *dst_sym, const void *src_local, size_t nbytes, uint64_t *sig_sym, uint64_t value, int pe)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    // both halves are checked before either is enqueued
    const uint64_t off = off_of(dst_sym), sig_off = off_of(sig_sym);
    if (int rc = hostlogic::check_contig(H.npes, H.seg, pe_self, pe, off, nbytes)) return rc;
    if (int rc = hostlogic::check_amo(H.npes, H.seg, pe_self, pe, sig_off)) return rc;
    if (nbytes && !src_local) return SHMEM_ERR_INVALID_ARG;
    if (nbytes)
        if (int rc = launch_copy(H.heap + (size_t)pe * H.seg + off, (const uint8_t *)src_local, nbytes)) return rc;
    // the add is a launch of its own behind the copy: the kernel boundary makes the data visible first
    return amo_single(SHMEM_AMO_FETCH_ADD, pe_self, sig_sym, value, 0, pe, nullptr);
}

int shmem_atomic_fetch_add(int pe_self, uint64_t *dst_sym, uint64_t value, int pe, uint64_t *dev_result)
{
    return amo_single(SHMEM_AMO_FETCH_ADD, pe_self, dst_sym, value, 0, pe, dev_result);
}
int shmem_atomic_compare_swap(int pe_self, uint64_t *dst_sym, uint64_t cond, uint64_t value, int pe, uint64_t *dev_result)
{
    return amo_single(SHMEM_AMO_COMPARE_SWAP, pe_self, dst_sym, cond, value, pe, dev_result);
}
int shmem_atomic_fetch_or(int pe_self, uint64_t *dst_sym, uint64_t value, int pe, uint64_t *dev_result)
{
    return amo_single(SHMEM_AMO_FETCH_OR, pe_self, dst_sym, value, 0, pe, dev_result);
}

int shmem_fence(int pe_self)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    return pe_ok(pe_self) ? SHMEM_OK : SHMEM_ERR_INVALID_PE;
}
int shmem_quiet(int pe_self)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    return (pe_self == -1 || pe_ok(pe_self)) ? SHMEM_OK : SHMEM_ERR_INVALID_PE;
}
int shmem_barrier_all(void) { return H.init ? SHMEM_OK : SHMEM_ERR_NOT_INIT; }

int shmem_stream_sync(uint64_t *first_bad_index)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (hipMemcpyAsync(H.pinned, H.scratch, 16, hipMemcpyDeviceToHost, H.stream) != hipSuccess) return SHMEM_ERR_DEVICE;
    if (hipStreamSynchronize(H.stream) != hipSuccess) return SHMEM_ERR_DEVICE;
    if (H.pinned[0] == 0) return SHMEM_OK;
    if (first_bad_index) *first_bad_index = H.pinned[1];
    if (H.pinned[0] == shmemx::DEV_ERR_BARRIER_TIMEOUT) {
        // A bounded wait gave up: arrival counts and generations of whatever barrier or signal wait was under
        // way are half-advanced, and every later barrier on them would miscount.  Nothing runs on the stream
        // now, so all synchronisation state starts again from zero: the scratch words, and the signal, counter
        // and barrier words of every live Gin, team and MoE object.
        if (hipMemsetAsync(H.scratch, 0, shmem_scratch_bytes(H.npes), H.stream) != hipSuccess) return SHMEM_ERR_DEVICE;
        std::vector<shmemx::GinState> words;
        {
            std::lock_guard<std::mutex> lk(H.mu);
            words = H.sync_words;
        }
        for (const shmemx::GinState &g : words)
            hipLaunchKernelGGL(shmemx::k_gin_zero, dim3((unsigned)std::min(H.npes, 1024)), dim3(256), 0, H.stream, ctx(), g);
        if (hipStreamSynchronize(H.stream) != hipSuccess) return SHMEM_ERR_DEVICE;
    } else if (hipMemsetAsync(H.scratch, 0, 16, H.stream) != hipSuccess) {
        return SHMEM_ERR_DEVICE;
    }
    return SHMEM_ERR_DEVICE_FAULT;
}

// ---------------------------------------------------------------------------
int shmem_op_batch(const void *dev_ops, size_t n, size_t quiet_every, int wgs_per_pe)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!grid_fits(wgs_per_pe) || (n && !dev_ops) || (uintptr_t)dev_ops % 8) return SHMEM_ERR_INVALID_ARG;
    if (n == 0) return SHMEM_OK;
    long grid = (long)H.npes * wgs_per_pe;
    // teams of 16 workgroups and more are bandwidth configurations: their large ops stream
    auto kernel = wgs_per_pe >= 16 ? shmemx::k_op_batch<true> : shmemx::k_op_batch<false>;
    if (grid > max_resident_wgs(kernel)) return SHMEM_ERR_INVALID_ARG;
    shmemx::Ctx c = ctx();
    const shmem_op_desc *ops = (const shmem_op_desc *)dev_ops;
    void *args[] = {&c, &ops, &n, &quiet_every, &wgs_per_pe};
    return launch_resident((const void *)kernel, dim3((unsigned)grid), dim3(WG_THREADS), args);
}

int shmem_op_batch_noalloc(int npes, size_t heap_bytes_per_pe, void *dev_heap, const void *dev_ops, size_t n,
                           size_t quiet_every, int wgs_per_pe, uint64_t *dev_fault, void *hip_stream)
{
    if (npes < 1 || heap_bytes_per_pe == 0 || !dev_heap || (n && !dev_ops) || wgs_per_pe < 1 || (uintptr_t)dev_ops % 8 ||
        (uintptr_t)dev_fault % 8) return SHMEM_ERR_INVALID_ARG;
    if (npes > NOALLOC_MAX_PES) return SHMEM_ERR_OUT_OF_RANGE;       // beyond what the built-in scratch words cover
    if (heap_bytes_per_pe % GRAN || (uintptr_t)dev_heap % GRAN) return SHMEM_ERR_ALIGN;
    if (heap_bytes_per_pe > SIZE_MAX / (size_t)npes) return SHMEM_ERR_INVALID_ARG;
    NoallocDevice *d = nullptr;
    if (int rc = noalloc_setup(&d)) return rc;
    const long grid = (long)npes * wgs_per_pe;
    const bool stream_inst = wgs_per_pe >= 16;
    if (grid > (stream_inst ? d->resident_stream : d->resident_small)) return SHMEM_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)hip_stream;
    // every call on a GPU shares that GPU's words and finds what the last call left: clear the ones this
    // launch uses (a fill kernel, not a memset node, so that the sequence can be captured into a graph)
    const uint32_t words = (uint32_t)(shmemx::W_PE_BASE + (size_t)npes * shmemx::W_PE_WORDS);
    hipLaunchKernelGGL(k_fill_zero, dim3((words + 255) / 256), dim3(256), 0, st, d->ptr, words);
    if (int rc = launched()) return rc;
    if (n) {
        shmemx::Ctx c{(uint8_t *)dev_heap, (uint64_t)heap_bytes_per_pe, d->ptr, npes};
        const shmem_op_desc *ops = (const shmem_op_desc *)dev_ops;
        void *args[] = {&c, &ops, &n, &quiet_every, &wgs_per_pe};
        const void *kernel = stream_inst ? (const void *)shmemx::k_op_batch<true> : (const void *)shmemx::k_op_batch<false>;
        if (hipLaunchKernel(kernel, dim3((unsigned)grid), dim3(WG_THREADS), args, 0, st) != hipSuccess) return SHMEM_ERR_DEVICE;
    }
    if (dev_fault) {
        hipLaunchKernelGGL(k_fault_out, dim3(1), dim3(64), 0, st, (const uint64_t *)d->ptr, dev_fault);
        if (int rc = launched()) return rc;
    }
    return SHMEM_OK;
}

int shmem_copy_sweep(int kind, void *remote_sym, void *local_sym, size_t count, size_t elem_bytes,
                     ptrdiff_t remote_stride, ptrdiff_t local_stride, size_t remote_slot_bytes,
                     size_t local_slot_bytes, size_t nslots, int ops_per_pe, int wgs_per_pe)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (kind < SHMEM_OP_PUT || kind > SHMEM_OP_IGET || !grid_fits(wgs_per_pe) || ops_per_pe < 0 || nslots < 1) return SHMEM_ERR_INVALID_ARG;
    const bool is_strided = kind >= SHMEM_OP_IPUT;
    uint64_t rspan = count, lspan = count;
    if (is_strided) {
        if (elem_bytes != 1 && elem_bytes != 2 && elem_bytes != 4 && elem_bytes != 8) return SHMEM_ERR_INVALID_ARG;
        if (remote_stride < 1 || local_stride < 1) return SHMEM_ERR_INVALID_ARG;
        if ((uintptr_t)remote_sym % elem_bytes || (uintptr_t)local_sym % elem_bytes ||
            remote_slot_bytes % elem_bytes || local_slot_bytes % elem_bytes) return SHMEM_ERR_ALIGN;
        if (!strided_span(count, remote_stride, elem_bytes, &rspan) ||
            !strided_span(count, local_stride, elem_bytes, &lspan)) return SHMEM_ERR_OUT_OF_RANGE;
    } else {
        elem_bytes = 1; remote_stride = local_stride = 1;
    }
    if (nslots > 1 && (rspan > remote_slot_bytes || lspan > local_slot_bytes)) return SHMEM_ERR_INVALID_ARG;
    unsigned __int128 rtot = (unsigned __int128)(nslots - 1) * remote_slot_bytes + rspan;
    unsigned __int128 ltot = (unsigned __int128)(nslots - 1) * local_slot_bytes + lspan;
    if (rtot > H.seg || ltot > H.seg) return SHMEM_ERR_OUT_OF_RANGE;
    uint64_t roff, loff;
    if (int rc = sym_off(remote_sym, (uint64_t)rtot, &roff)) return rc;
    if (int rc = sym_off(local_sym, (uint64_t)ltot, &loff)) return rc;
    // the local and the remote window of one segment must not intersect (PE p's
    // remote window is written/read by PE p-1 while p uses its local window)
    if (roff < loff + (uint64_t)ltot && loff < roff + (uint64_t)rtot) return SHMEM_ERR_INVALID_ARG;
    if (count == 0 || ops_per_pe == 0) return SHMEM_OK;
    shmemx::SweepArgs a;
    a.kind = kind; a.remote_off = roff; a.local_off = loff; a.count = count; a.elem_bytes = (uint32_t)elem_bytes;
    a.remote_stride = remote_stride; a.local_stride = local_stride; a.remote_slot = remote_slot_bytes;
    a.local_slot = local_slot_bytes; a.nslots = nslots; a.ops_per_pe = (uint32_t)ops_per_pe;
    a.wgs_per_pe = (uint32_t)wgs_per_pe;
    uint32_t team = 0;
    if (const int how = sweep_stream_kind(is_strided, count, remote_slot_bytes, local_slot_bytes, roff, loff, nslots, ops_per_pe,
                                          wgs_per_pe, &team)) {
        shmemx::StreamSweepArgs sa;
        sa.kind = kind; sa.remote_off = roff; sa.local_off = loff; sa.count = count;
        sa.remote_slot = remote_slot_bytes; sa.local_slot = local_slot_bytes; sa.nslots = (uint32_t)nslots;
        sa.ops_per_pe = (uint32_t)ops_per_pe; sa.team = team;
        const unsigned grid = (unsigned)H.npes * team;
        sa.period = stream_period(grid);
        if (how == 1)
            hipLaunchKernelGGL(shmemx::k_copy_sweep_stream_dyn, dim3(grid), dim3(shmemx::ST_DYN_THREADS), 0, H.stream, ctx(), sa);
        else if (how == 3)
            hipLaunchKernelGGL(shmemx::k_copy_sweep_stream_rows, dim3(grid), dim3(shmemx::ST_DYN_THREADS), 0, H.stream, ctx(), sa);
        else if (how == 4)
            hipLaunchKernelGGL(shmemx::k_copy_sweep_stream_packed, dim3(grid), dim3(shmemx::ST_DYN_THREADS), 0, H.stream, ctx(), sa);
        else
            hipLaunchKernelGGL(shmemx::k_copy_sweep_stream, dim3(grid), dim3(shmemx::ST_THREADS), 0, H.stream, ctx(), sa);
        return launched();
    }
    hipLaunchKernelGGL(shmemx::k_copy_sweep, dim3((unsigned)(H.npes * wgs_per_pe)), dim3(WG_THREADS), 0, H.stream,
                       ctx(), a);
    return launched();
}

int shmem_copy_sweep_geometry(int kind, void *remote_sym, void *local_sym, size_t count, size_t remote_slot_bytes,
                              size_t local_slot_bytes, size_t nslots, int ops_per_pe, int wgs_per_pe, int *workgroups_out,
                              int *threads_out)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (kind < SHMEM_OP_PUT || kind > SHMEM_OP_IGET || !grid_fits(wgs_per_pe) || ops_per_pe < 0 || nslots < 1) return SHMEM_ERR_INVALID_ARG;
    uint32_t team = 0;
    const int how = sweep_stream_kind(kind >= SHMEM_OP_IPUT, count, remote_slot_bytes, local_slot_bytes, off_of(remote_sym),
                                      off_of(local_sym), nslots, ops_per_pe, wgs_per_pe, &team);
    if (workgroups_out) *workgroups_out = how ? H.npes * (int)team : H.npes * wgs_per_pe;
    if (threads_out) *threads_out = how == 1 || how == 3 || how == 4 ? (int)shmemx::ST_DYN_THREADS : how == 2 ? (int)shmemx::ST_THREADS : WG_THREADS;
    return SHMEM_OK;
}

int shmem_amo_batch(int kind, uint64_t *ctr_sym, size_t T, const int32_t *dev_pe, const uint32_t *dev_idx,
                    const uint64_t *dev_a, const uint64_t *dev_b, uint64_t *dev_old, size_t n,
                    int wgs_per_pe, int aggregate)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (kind < SHMEM_AMO_FETCH_ADD || kind > SHMEM_AMO_MIN_CAS_LOOP || !grid_fits(wgs_per_pe) || T == 0) return SHMEM_ERR_INVALID_ARG;
    if (T > H.seg / 8) return SHMEM_ERR_OUT_OF_RANGE;
    if ((uintptr_t)ctr_sym % 8) return SHMEM_ERR_ALIGN;
    uint64_t off;
    if (int rc = sym_off(ctr_sym, (uint64_t)T * 8, &off)) return rc;
    if (n == 0) return SHMEM_OK;
    if (!dev_pe || !dev_idx || !dev_a || (kind == SHMEM_AMO_COMPARE_SWAP && !dev_b)) return SHMEM_ERR_INVALID_ARG;
    shmemx::AmoArgs a;
    a.kind = kind; a.ctr_off = off; a.T = T; a.pe = dev_pe; a.idx = dev_idx; a.a = dev_a; a.b = dev_b;
    a.old = dev_old; a.n = n; a.per_pe = (n + (size_t)H.npes - 1) / (size_t)H.npes; a.wgs_per_pe = (uint32_t)wgs_per_pe;
    dim3 grid((unsigned)(H.npes * wgs_per_pe)), block(WG_THREADS);
    // the combining kernel keys its LDS table by pe * T + idx in 32 bits
    const bool agg = aggregate && kind != SHMEM_AMO_COMPARE_SWAP && (uint64_t)H.npes * T < 0xFFFFFFFFull;
    if (agg) hipLaunchKernelGGL(shmemx::k_amo_batch_agg, grid, block, 0, H.stream, ctx(), a);
    else hipLaunchKernelGGL(shmemx::k_amo_batch, grid, block, 0, H.stream, ctx(), a);
    return launched();
}

static int hash_common(const uint64_t *table_sym, size_t slots, const uint64_t *keys, size_t n, int wgs, uint64_t *off)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (slots == 0 || !grid_fits(wgs) || slots > UINT32_MAX) return SHMEM_ERR_INVALID_ARG;
    if (slots > H.seg / 8) return SHMEM_ERR_OUT_OF_RANGE;
    if ((uintptr_t)table_sym % 8) return SHMEM_ERR_ALIGN;
    if (int rc = sym_off(table_sym, (uint64_t)slots * 8, off)) return rc;
    if (n && !keys) return SHMEM_ERR_INVALID_ARG;
    return SHMEM_OK;
}

int shmem_hash_insert(uint64_t *table_sym, size_t slots_per_pe, const uint64_t *dev_keys, size_t n,
                      uint8_t *dev_status, int wgs_per_pe)
{
    uint64_t off;
    if (int rc = hash_common(table_sym, slots_per_pe, dev_keys, n, wgs_per_pe, &off)) return rc;
    if (n == 0) return SHMEM_OK;
    shmemx::HashArgs a{off, (uint32_t)slots_per_pe, dev_keys, n, (n + (size_t)H.npes - 1) / (size_t)H.npes,
                       dev_status, (uint32_t)wgs_per_pe};
    hipLaunchKernelGGL(shmemx::k_hash_insert, dim3((unsigned)(H.npes * wgs_per_pe)), dim3(WG_THREADS), 0, H.stream,
                       ctx(), a);
    return launched();
}

int shmem_hash_lookup(const uint64_t *table_sym, size_t slots_per_pe, const uint64_t *dev_keys, size_t n,
                      uint8_t *dev_found, int wgs_per_pe)
{
    uint64_t off;
    if (int rc = hash_common(table_sym, slots_per_pe, dev_keys, n, wgs_per_pe, &off)) return rc;
    if (n == 0) return SHMEM_OK;
    if (!dev_found) return SHMEM_ERR_INVALID_ARG;
    shmemx::HashArgs a{off, (uint32_t)slots_per_pe, dev_keys, n, (n + (size_t)H.npes - 1) / (size_t)H.npes,
                       dev_found, (uint32_t)wgs_per_pe};
    const dim3 grid((unsigned)(H.npes * wgs_per_pe));
    if (slots_per_pe % shmemx::HASH_SECTOR == 0 && off % 64 == 0)     // whole, aligned 64-byte sectors
        hipLaunchKernelGGL(shmemx::k_hash_lookup_sectors<HASH_LOOKUP_KIF>, grid, dim3(WG_THREADS), 0, H.stream, ctx(), a);
    else
        hipLaunchKernelGGL(shmemx::k_hash_lookup, grid, dim3(WG_THREADS), 0, H.stream, ctx(), a);
    return launched();
}

// ---------------------------------------------------------------------------
int shmem_bfs_create(uint32_t nverts, const uint64_t *dev_row_off, const uint32_t *dev_nbr, int wgs_per_pe,
                     void **graph_out)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!graph_out || nverts == 0 || !dev_row_off || !grid_fits(wgs_per_pe)) return SHMEM_ERR_INVALID_ARG;
    BfsGraph *g = new (std::nothrow) BfsGraph();
    if (!g) return SHMEM_ERR_NOMEM;
    const uint32_t vpp = (uint32_t)(((uint64_t)nverts + (uint64_t)H.npes - 1) / (uint64_t)H.npes);
    const uint64_t words = ((uint64_t)vpp + 63) / 64;
    // bitmap, (parent, level) records, two queues, long-row list, its segment scan, counters, per-die bitmap
    // copies, frontier bitmap, previous-level bitmap, has-neighbours bitmap
    const size_t sizes[11] = {words * 8, (size_t)vpp * 8, (size_t)vpp * 4, (size_t)vpp * 4,
                              (size_t)vpp * 4, ((size_t)vpp + 1) * 4, 256, words * 8 * shmemx::NXCD, words * 8,
                              words * 8, words * 8};
    uint64_t offs[11];
    g->nallocs = 0;
    for (int i = 0; i < 11; ++i) {
        void *p = shmem_malloc(sizes[i]);
        if (!p) {
            for (int k = 0; k < g->nallocs; ++k) shmem_free(g->allocs[k]);
            delete g;
            return SHMEM_ERR_NOMEM;
        }
        g->allocs[g->nallocs++] = p;
        offs[i] = (uint64_t)((uint8_t *)p - H.heap);
    }
    shmemx::BfsState &s = g->st;
    auto fail = [&](int rc) {
        for (int k = 0; k < g->nallocs; ++k) shmem_free(g->allocs[k]);
        (void)hipFree(g->d_row_int); (void)hipFree(g->d_nbr_int); (void)hipFree(g->d_to_int); (void)hipFree(g->d_to_orig);
        delete g;
        return rc;
    };
    g->d_row_int = nullptr; g->d_nbr_int = nullptr; g->d_to_int = nullptr; g->d_to_orig = nullptr;
    const uint64_t nint64 = (uint64_t)vpp * (uint64_t)H.npes;               // every PE a full block (padded with vertices without edges)
    if (nint64 >= SHMEM_BFS_NONE) return fail(SHMEM_ERR_INVALID_ARG);
    const uint32_t nint = (uint32_t)nint64;
    s.nverts = nint; s.vpp = vpp; s.words = words;
    s.shift = (vpp & (vpp - 1)) == 0 ? (int)__builtin_ctz(vpp) : -1;
    // blocks of up to 4096 words (256 lines) inside which the claim bitmap spreads neighbouring words over lines
    s.vis_block_log2 = 0;
    if (words >= 32) {
        uint32_t lg = 63u - (uint32_t)__builtin_clzll((unsigned long long)words);
        s.vis_block_log2 = lg > 12 ? 12 : lg;
    }
    s.bitmap_off = offs[0]; s.pl_off = offs[1];
    s.queue_off[0] = offs[2]; s.queue_off[1] = offs[3]; s.big_off = offs[4]; s.bigscan_off = offs[5];
    s.tails_off = offs[6]; s.filter_off = offs[7]; s.front_off = offs[8]; s.prev_off = offs[9]; s.linked_off = offs[10];
    g->mode = SHMEM_BFS_TOP_DOWN; g->canonical = false; g->alpha = BFS_ALPHA; g->beta = BFS_BETA;
    g->nverts_orig = nverts;
    // The library's numbering: vertices ranked by degree, largest first (ties by number), rank r -> local vertex
    // r / npes of PE r mod npes.  Ranking and the new row offsets are host work, once per graph.
    try {
    std::vector<uint64_t> row((size_t)nverts + 1);
    if (hipMemcpyAsync(row.data(), dev_row_off, row.size() * 8, hipMemcpyDeviceToHost, H.stream) != hipSuccess ||
        hipStreamSynchronize(H.stream) != hipSuccess) return fail(SHMEM_ERR_DEVICE);
    g->nnz = row[nverts];
    if (g->nnz && !dev_nbr) return fail(SHMEM_ERR_INVALID_ARG);
    for (uint32_t v = 0; v < nverts; ++v) if (row[v + 1] < row[v]) return fail(SHMEM_ERR_INVALID_ARG);
    std::vector<uint32_t> order(nverts), to_orig(nint, SHMEM_BFS_NONE);
    for (uint32_t v = 0; v < nverts; ++v) order[v] = v;
    std::sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) {
        const uint64_t da = row[a + 1] - row[a], db = row[b + 1] - row[b];
        return da != db ? da > db : a < b;
    });
    g->to_int.assign(nverts, 0);
    g->n_long = 0;
    for (uint32_t r = 0; r < nverts; ++r) {
        if (row[order[r] + 1] - row[order[r]] >= shmemx::BIG_DEGREE) g->n_long = r + 1;
        const uint32_t i = (r % (uint32_t)H.npes) * vpp + r / (uint32_t)H.npes;
        g->to_int[order[r]] = i;
        to_orig[i] = order[r];
    }
    std::vector<uint32_t>().swap(order);
    std::vector<uint64_t> row_int((size_t)nint + 1);
    row_int[0] = 0;
    for (uint32_t i = 0; i < nint; ++i) {
        const uint32_t o = to_orig[i];
        row_int[i + 1] = row_int[i] + (o == SHMEM_BFS_NONE ? 0 : row[o + 1] - row[o]);
    }
    std::vector<uint64_t>().swap(row);
    if (hipMalloc((void **)&g->d_row_int, row_int.size() * 8) != hipSuccess || hipMalloc((void **)&g->d_nbr_int, std::max<uint64_t>(g->nnz, 1) * 4) != hipSuccess ||
        hipMalloc((void **)&g->d_to_int, (size_t)nverts * 4) != hipSuccess || hipMalloc((void **)&g->d_to_orig, (size_t)nint * 4) != hipSuccess)
        return fail(SHMEM_ERR_NOMEM);
    if (hipMemcpyAsync(g->d_row_int, row_int.data(), row_int.size() * 8, hipMemcpyHostToDevice, H.stream) != hipSuccess ||
        hipMemcpyAsync(g->d_to_int, g->to_int.data(), (size_t)nverts * 4, hipMemcpyHostToDevice, H.stream) != hipSuccess ||
        hipMemcpyAsync(g->d_to_orig, to_orig.data(), (size_t)nint * 4, hipMemcpyHostToDevice, H.stream) != hipSuccess)
        return fail(SHMEM_ERR_DEVICE);
    H.pinned[40] = 0;                                                        // set by the kernel if a neighbour is no vertex
    hipLaunchKernelGGL(shmemx::k_bfs_relabel, dim3((unsigned)std::max(1, H.num_cus) * 8), dim3(WG_THREADS), 0, H.stream, nint, nverts, vpp,
                       g->d_to_orig, g->d_to_int, dev_row_off, dev_nbr, g->d_row_int, g->d_nbr_int, H.pinned + 40);
    if (hipStreamSynchronize(H.stream) != hipSuccess) return fail(SHMEM_ERR_DEVICE);   // the host vectors above are done with
    if (__atomic_load_n(H.pinned + 40, __ATOMIC_ACQUIRE) != 0) return fail(SHMEM_ERR_INVALID_ARG);
    if (H.bfs_sort_rows && g->nnz > 0 && g->nnz < UINT32_MAX) {
        // Every row is then sorted by the degree rank of its neighbours, the best-connected first (a segmented radix
        // sort over the whole adjacency; the entries are turned into ranks and back around it).  The 64 neighbours that
        // one wave instruction probes are then next to each other in rank, i.e. at about the same local vertex of every
        // owner: one line of every owner's bitmap instead of up to 64 lines.  If the memory for it cannot be had, the
        // rows stay as the relabelling left them (in four classes of rank).
        uint32_t *sorted = nullptr;
        void *temp = nullptr;
        size_t temp_bytes = 0;
        unsigned bits = 1;
        while (bits < 32 && (1ull << bits) < nint64) ++bits;
        const dim3 kgrid((unsigned)std::max(1, H.num_cus) * 8), kblock(WG_THREADS);
        const uint64_t *row_begin = g->d_row_int, *row_end = g->d_row_int + 1;
        bool ok = hipMalloc((void **)&sorted, g->nnz * 4) == hipSuccess &&
                  rocprim::segmented_radix_sort_keys(nullptr, temp_bytes, g->d_nbr_int, sorted, (unsigned)g->nnz, (unsigned)nint,
                                                     row_begin, row_end, 0u, bits, H.stream) == hipSuccess &&
                  hipMalloc(&temp, std::max<size_t>(temp_bytes, 16)) == hipSuccess;
        if (ok) {
            hipLaunchKernelGGL(shmemx::k_bfs_rekey, kgrid, kblock, 0, H.stream, g->d_nbr_int, g->nnz, vpp, (uint32_t)H.npes, 1);
            ok = rocprim::segmented_radix_sort_keys(temp, temp_bytes, g->d_nbr_int, sorted, (unsigned)g->nnz, (unsigned)nint,
                                                    row_begin, row_end, 0u, bits, H.stream) == hipSuccess;
            hipLaunchKernelGGL(shmemx::k_bfs_rekey, kgrid, kblock, 0, H.stream, ok ? sorted : g->d_nbr_int, g->nnz, vpp, (uint32_t)H.npes, 0);
            if (hipStreamSynchronize(H.stream) != hipSuccess) { (void)hipFree(temp); (void)hipFree(sorted); return fail(SHMEM_ERR_DEVICE); }
        }
        if (temp) (void)hipFree(temp);
        if (ok) { (void)hipFree(g->d_nbr_int); g->d_nbr_int = sorted; }
        else {
            if (sorted) (void)hipFree(sorted);
            (void)hipGetLastError();
        }
    }
    } catch (const std::bad_alloc &) {
        return fail(SHMEM_ERR_NOMEM);
    }
    s.row_off = g->d_row_int; s.nbr = g->d_nbr_int; s.to_orig = g->d_to_orig;
    s.wgs_per_pe = (uint32_t)wgs_per_pe;     // before any launch that takes the state
    g->wgs_per_pe = wgs_per_pe;
    hipLaunchKernelGGL(shmemx::k_bfs_mark_linked, dim3((unsigned)(H.npes * wgs_per_pe)), dim3(WG_THREADS), 0, H.stream,
                       ctx(), g->st);
    if (int rc = launched()) return fail(rc);
    *graph_out = g;
    return SHMEM_OK;
}

int shmem_bfs_destroy(void *graph)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!graph) return SHMEM_ERR_INVALID_ARG;
    BfsGraph *g = (BfsGraph *)graph;
    int rc = SHMEM_OK;
    for (int k = 0; k < g->nallocs; ++k) if (shmem_free(g->allocs[k]) != SHMEM_OK) rc = SHMEM_ERR_BAD_FREE;
    if (hipStreamSynchronize(H.stream) != hipSuccess) rc = SHMEM_ERR_DEVICE;     // nothing in flight reads the graph any more
    (void)hipFree(g->d_row_int); (void)hipFree(g->d_nbr_int); (void)hipFree(g->d_to_int); (void)hipFree(g->d_to_orig);
    delete g;
    return rc;
}

int shmem_bfs_configure(void *graph, int mode, int alpha, int beta)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    const int direction = mode & ~SHMEM_BFS_CANONICAL_PARENTS;
    if (!graph || direction < SHMEM_BFS_TOP_DOWN || direction > SHMEM_BFS_BOTTOM_UP || alpha < 0 || beta < 0)
        return SHMEM_ERR_INVALID_ARG;
    BfsGraph *g = (BfsGraph *)graph;
    g->mode = direction;
    g->canonical = (mode & SHMEM_BFS_CANONICAL_PARENTS) != 0;
    g->alpha = alpha ? (uint32_t)alpha : BFS_ALPHA;
    g->beta = beta ? (uint32_t)beta : BFS_BETA;
    return SHMEM_OK;
}

int shmem_bfs(void *graph, uint32_t root, int32_t *dev_level, uint32_t *dev_parent, shmem_bfs_stats *stats)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!graph) return SHMEM_ERR_INVALID_ARG;
    BfsGraph *g = (BfsGraph *)graph;
    const shmemx::BfsState &s = g->st;
    if (root >= g->nverts_orig) return SHMEM_ERR_INVALID_ARG;
    const uint32_t nverts = g->nverts_orig;
    root = g->to_int[root];                                                  // the search runs on the library's numbering
    g->last_levels = 0;
    shmemx::Ctx c = ctx();
    dim3 grid((unsigned)(H.npes * g->wgs_per_pe)), block(WG_THREADS);
    shmem_bfs_stats st;
    memset(&st, 0, sizeof st);
    const bool staged = H.npes <= (int)shmemx::STAGE_PES;   // winners staged in LDS per owner
    const bool hybrid = g->mode != SHMEM_BFS_TOP_DOWN;
    // [0] size of the next frontier, [1] degree sum of the expanded frontiers (top-down only mode),
    // [2] running degree sum of every frontier discovered so far (direction-optimising modes)
    uint64_t *counts = H.pinned + 16;
    // Frontiers of at least nverts / sort_div vertices are expanded from a queue in vertex order (rewritten from
    // the level's new bits); the frontier bitmap is then kept level by level in top-down searches as well.
    const uint64_t sort_from = H.bfs_sort_div ? std::max<uint64_t>(nverts / H.bfs_sort_div, 1024) : UINT64_MAX;
    const bool fronts = hybrid || H.bfs_sort_div != 0;
    // The start also leaves what a level end would: the root as the frontier bitmap and as the previous level's
    // snapshot, its row length as the first degree sum (direction-optimising modes) and, for the host, in counts[4],
    // which is read after the first level (its hand-over orders the two).  Level 0 therefore runs top-down in the
    // direction-optimising mode whatever the root's degree: its frontier is one vertex.
    hipLaunchKernelGGL(shmemx::k_bfs_init, grid, block, 0, H.stream, c, s, root, (int)fronts, (int)hybrid, counts + 4);
    uint64_t n_f = 1, n_f_prev = 0, m_f = 0, cum_mf = 0;
    const uint32_t root_rank = (root % s.vpp) * (uint32_t)H.npes + root / s.vpp;
    st.frontier_size[0] = 1;
    st.reached = 1;
    bool bottom_up = false;
    bool queue_written = true;   // the frontier's queue exists (a bottom-up level only counts its finds)
    uint32_t L = 0;
    auto t_level = std::chrono::steady_clock::now();
    for (;;) {
        if (g->mode == SHMEM_BFS_BOTTOM_UP) bottom_up = true;
        else if (g->mode == SHMEM_BFS_DIRECTION_OPTIMIZING) {
            // switch when the frontier's edges outweigh a fraction of the edges still hanging off
            // unvisited vertices; switch back when the frontier is small and shrinking
            const uint64_t m_u = g->nnz > cum_mf ? g->nnz - cum_mf : 0;
            if (!bottom_up) bottom_up = m_f > m_u / g->alpha;
            else if (n_f < nverts / g->beta && n_f < n_f_prev) bottom_up = false;
        }
        if (!bottom_up && !queue_written) {
            hipLaunchKernelGGL(shmemx::k_bfs_fill_queue, grid, block, 0, H.stream, c, s, L);   // from the frontier bitmap
            queue_written = true;
        } else if (!bottom_up && L > 0 && n_f >= sort_from) {
            hipLaunchKernelGGL(shmemx::k_bfs_fill_queue, grid, block, 0, H.stream, c, s, L);   // the same entries, in vertex order
        }
        if (bottom_up) {
            // no LDS and few registers: twice the workgroups per PE fill the CUs' wave slots
            shmemx::BfsState s2 = s;
            s2.wgs_per_pe = s.wgs_per_pe * 2;
            hipLaunchKernelGGL(shmemx::k_bfs_bottomup, dim3(grid.x * 2), block, 0, H.stream, c, s2, L);
            queue_written = false;
        } else {
            // the long-row pass is left out where the host can tell that the frontier has no long row: the root by
            // its rank, a later frontier by its degree sum (known in the direction-optimising modes) -- the first and
            // the last levels of a search, which are little more than their launches
            const bool no_long = g->n_long == 0 || (L == 0 ? root_rank >= g->n_long : (hybrid && m_f < shmemx::BIG_DEGREE));
            if (staged) hipLaunchKernelGGL(shmemx::k_bfs_expand<true>, grid, block, 0, H.stream, c, s, L);
            else hipLaunchKernelGGL(shmemx::k_bfs_expand<false>, grid, block, 0, H.stream, c, s, L);
            if (!no_long) {
                hipLaunchKernelGGL(shmemx::k_bfs_bigscan, dim3((unsigned)H.npes), dim3(1024), 0, H.stream, c, s);
                if (staged) hipLaunchKernelGGL(shmemx::k_bfs_big<true>, grid, block, 0, H.stream, c, s, L);
                else hipLaunchKernelGGL(shmemx::k_bfs_big<false>, grid, block, 0, H.stream, c, s, L);
            }
        }
        if (int rc = bfs_level_end(s, L + 1, fronts, hybrid && !bottom_up, g->wgs_per_pe, counts)) return rc;
        if (L < 64) {
            const auto t_now = std::chrono::steady_clock::now();
            g->last_level_us[L] = std::chrono::duration<float, std::micro>(t_now - t_level).count();
            g->last_level_bottom_up[L] = bottom_up ? 1 : 0;
            t_level = t_now;
        }
        ++L;
        if (counts[0] == 0) break;
        if (L >= (uint32_t)INT32_MAX) return SHMEM_ERR_INVALID_ARG;   // levels are int32
        if (L < 64) st.frontier_size[L] = counts[0];
        st.reached += counts[0];
        n_f_prev = n_f; n_f = counts[0];
        if (hybrid) {
            if (L == 1) cum_mf = counts[4];          // the root's row length, written by the start of the search
            m_f = counts[2] - cum_mf; cum_mf = counts[2];
        }
    }
    st.nlevels = L;
    g->last_levels = L < 64 ? L : 64;
    st.edges_traversed = (hybrid ? counts[2] : counts[1]) / 2;
    if (g->canonical) hipLaunchKernelGGL(shmemx::k_bfs_canonical, grid, block, 0, H.stream, c, s);
    if (dev_level || dev_parent) {
        hipLaunchKernelGGL(shmemx::k_bfs_gather, grid, block, 0, H.stream, c, s, nverts, g->d_to_int, dev_level, dev_parent);
        if (hipStreamSynchronize(H.stream) != hipSuccess) return SHMEM_ERR_DEVICE;
    }
    if (stats) *stats = st;
    return launched();
}

int shmem_bfs_level_times(void *graph, uint32_t *nlevels_out, float *us_out, uint8_t *bottom_up_out, uint32_t max_levels)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!graph || !nlevels_out) return SHMEM_ERR_INVALID_ARG;
    const BfsGraph *g = (const BfsGraph *)graph;
    const uint32_t n = std::min(g->last_levels, max_levels);
    *nlevels_out = n;
    for (uint32_t i = 0; i < n; ++i) {
        if (us_out) us_out[i] = g->last_level_us[i];
        if (bottom_up_out) bottom_up_out[i] = g->last_level_bottom_up[i];
    }
    return SHMEM_OK;
}

// ---------------------------------------------------------------------------
struct GinObj { shmemx::GinState st; void *alloc; };

int shmem_gin_create(int nsignals, int ncounters, void **gin_out)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!gin_out || nsignals < 1 || ncounters < 0 || nsignals > (1 << 20) || ncounters > (1 << 20)) return SHMEM_ERR_INVALID_ARG;
    GinObj *g = new (std::nothrow) GinObj();
    if (!g) return SHMEM_ERR_NOMEM;
    const size_t sig_bytes = ((size_t)nsignals * 8 + 255) / 256 * 256;
    g->alloc = shmem_malloc(sig_bytes + (size_t)std::max(ncounters, 1) * 8);
    if (!g->alloc) { delete g; return SHMEM_ERR_NOMEM; }
    g->st.signals_off = (uint64_t)((uint8_t *)g->alloc - H.heap);
    g->st.counters_off = g->st.signals_off + sig_bytes;
    g->st.nsignals = (uint32_t)nsignals; g->st.ncounters = (uint32_t)ncounters;
    hipLaunchKernelGGL(shmemx::k_gin_zero, dim3((unsigned)std::min(H.npes, 1024)), dim3(256), 0, H.stream, ctx(), g->st);
    if (int rc = launched()) { shmem_free(g->alloc); delete g; return rc; }
    sync_words_add(g->st);
    *gin_out = g;
    return SHMEM_OK;
}

int shmem_gin_destroy(void *gin)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!gin) return SHMEM_ERR_INVALID_ARG;
    GinObj *g = (GinObj *)gin;
    sync_words_remove(g->st);
    int rc = shmem_free(g->alloc);
    delete g;
    return rc;
}

void *shmem_gin_signal_sym(void *gin, int id)
{
    if (!H.init || !gin) return nullptr;
    GinObj *g = (GinObj *)gin;
    if (id < 0 || (uint32_t)id >= g->st.nsignals) return nullptr;
    return H.heap + g->st.signals_off + 8ull * (uint32_t)id;
}

void *shmem_gin_counter_sym(void *gin, int id)
{
    if (!H.init || !gin) return nullptr;
    GinObj *g = (GinObj *)gin;
    if (id < 0 || (uint32_t)id >= g->st.ncounters) return nullptr;
    return H.heap + g->st.counters_off + 8ull * (uint32_t)id;
}

// the two structs of the header are the kernels' own argument structs, field for field
static_assert(sizeof(shmem_device_ctx) == sizeof(shmemx::Ctx) && offsetof(shmem_device_ctx, heap) == offsetof(shmemx::Ctx, heap) &&
              offsetof(shmem_device_ctx, seg) == offsetof(shmemx::Ctx, seg) && offsetof(shmem_device_ctx, scratch) == offsetof(shmemx::Ctx, scratch) &&
              offsetof(shmem_device_ctx, npes) == offsetof(shmemx::Ctx, npes), "shmem_device_ctx must match shmemx::Ctx");
static_assert(sizeof(shmem_gin_state) == sizeof(shmemx::GinState) && offsetof(shmem_gin_state, counters_off) == offsetof(shmemx::GinState, counters_off) &&
              offsetof(shmem_gin_state, nsignals) == offsetof(shmemx::GinState, nsignals) &&
              offsetof(shmem_gin_state, ncounters) == offsetof(shmemx::GinState, ncounters), "shmem_gin_state must match shmemx::GinState");

int shmem_device_context(shmem_device_ctx *ctx_out)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!ctx_out) return SHMEM_ERR_INVALID_ARG;
    const shmemx::Ctx c = ctx();
    memcpy(ctx_out, &c, sizeof c);
    return SHMEM_OK;
}

int shmem_gin_device_state(void *gin, shmem_gin_state *state_out)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!gin || !state_out) return SHMEM_ERR_INVALID_ARG;
    memcpy(state_out, &((GinObj *)gin)->st, sizeof(shmemx::GinState));
    return SHMEM_OK;
}

int shmem_ring_exchange(void *recv_sym, const void *send_sym, size_t slot_bytes, void *gin, int signal_id,
                        int counter_id, int rounds, int wgs_per_pe)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!gin || rounds < 0 || !grid_fits(wgs_per_pe)) return SHMEM_ERR_INVALID_ARG;
    GinObj *g = (GinObj *)gin;
    if (signal_id < 0 || (uint32_t)signal_id >= g->st.nsignals || counter_id < 0 ||
        (uint32_t)counter_id >= g->st.ncounters) return SHMEM_ERR_INVALID_ARG;
    unsigned __int128 span = (unsigned __int128)slot_bytes * (unsigned)H.npes;
    if (span > H.seg) return SHMEM_ERR_OUT_OF_RANGE;
    uint64_t roff, soff;
    if (int rc = sym_off(recv_sym, (uint64_t)span, &roff)) return rc;
    if (int rc = sym_off(send_sym, (uint64_t)span, &soff)) return rc;
    if (roff < soff + (uint64_t)span && soff < roff + (uint64_t)span && span) return SHMEM_ERR_INVALID_ARG;
    if (rounds == 0) return SHMEM_OK;
    long grid = (long)H.npes * wgs_per_pe;
    if (grid > max_resident_wgs(shmemx::k_ring_exchange)) return SHMEM_ERR_INVALID_ARG;
    shmemx::Ctx c = ctx();
    shmemx::GinState gs = g->st;
    uint64_t ds = slot_bytes;
    uint32_t sig = (uint32_t)signal_id, ctr = (uint32_t)counter_id, r = (uint32_t)rounds, w = (uint32_t)wgs_per_pe;
    void *args[] = {&c, &gs, &roff, &soff, &ds, &sig, &ctr, &r, &w};
    return launch_resident((const void *)shmemx::k_ring_exchange, dim3((unsigned)grid), dim3(WG_THREADS), args);
}

int shmem_pingpong(void *buf_sym, size_t nbytes, void *gin, int signal_id, int iters)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!gin || H.npes < 2 || iters < 0) return SHMEM_ERR_INVALID_ARG;
    GinObj *g = (GinObj *)gin;
    if (signal_id < 0 || (uint32_t)signal_id >= g->st.nsignals) return SHMEM_ERR_INVALID_ARG;
    const uint64_t padded = ((uint64_t)nbytes + 255) / 256 * 256;
    if (padded > H.seg / 2) return SHMEM_ERR_OUT_OF_RANGE;
    uint64_t boff;
    if (int rc = sym_off(buf_sym, 2 * padded, &boff)) return rc;
    if (iters == 0) return SHMEM_OK;
    if (2 > max_resident_wgs(shmemx::k_pingpong)) return SHMEM_ERR_DEVICE;
    shmemx::Ctx c = ctx();
    shmemx::GinState gs = g->st;
    uint64_t nb = nbytes;
    uint32_t sig = (uint32_t)signal_id, it = (uint32_t)iters;
    void *args[] = {&c, &gs, &boff, &nb, &sig, &it};
    return launch_resident((const void *)shmemx::k_pingpong, dim3(2), dim3(WG_THREADS), args);
}

int shmem_barrier_epochs(uint64_t *slots_sym, int rounds, int wgs_per_pe, uint64_t *dev_errors)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (rounds < 0 || !grid_fits(wgs_per_pe)) return SHMEM_ERR_INVALID_ARG;
    if ((uintptr_t)slots_sym % 8 || (uintptr_t)dev_errors % 8) return SHMEM_ERR_ALIGN;
    uint64_t off;
    if (int rc = sym_off(slots_sym, 8ull * (uint64_t)H.npes, &off)) return rc;
    if (rounds == 0) return SHMEM_OK;
    long grid = (long)H.npes * wgs_per_pe;
    if (grid > max_resident_wgs(shmemx::k_barrier_epochs)) return SHMEM_ERR_INVALID_ARG;
    shmemx::Ctx c = ctx();
    uint32_t r = (uint32_t)rounds, w = (uint32_t)wgs_per_pe;
    void *args[] = {&c, &off, &r, &w, &dev_errors};
    return launch_resident((const void *)shmemx::k_barrier_epochs, dim3((unsigned)grid), dim3(WG_THREADS), args);
}

// ---------------------------------------------------------------------------
struct shmem_team { shmemx::PeTeam st; void *alloc; };

static_assert(sizeof(shmem_pe_team) == sizeof(shmemx::PeTeam) && offsetof(shmem_pe_team, stride) == offsetof(shmemx::PeTeam, stride) &&
              offsetof(shmem_pe_team, size) == offsetof(shmemx::PeTeam, size) && offsetof(shmem_pe_team, words_off) == offsetof(shmemx::PeTeam, words_off),
              "shmem_pe_team must match shmemx::PeTeam");

int shmem_team_create(int start, int stride, int size, shmem_team_t *team_out)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!team_out || start < 0 || stride < 1 || size < 1) return SHMEM_ERR_INVALID_ARG;
    if ((long long)start + (long long)(size - 1) * stride >= H.npes) return SHMEM_ERR_INVALID_PE;
    shmem_team *t = new (std::nothrow) shmem_team();
    if (!t) return SHMEM_ERR_NOMEM;
    t->alloc = shmem_malloc(256);
    if (!t->alloc) { delete t; return SHMEM_ERR_NOMEM; }
    t->st = shmemx::PeTeam{(uint32_t)start, (uint32_t)stride, (uint32_t)size, 0u, (uint64_t)((uint8_t *)t->alloc - H.heap)};
    // arrivals and generation start at zero on every PE (only the first member's copy is used)
    shmemx::GinState z{t->st.words_off, t->st.words_off, 32u, 0u};
    hipLaunchKernelGGL(shmemx::k_gin_zero, dim3((unsigned)std::min(H.npes, 1024)), dim3(256), 0, H.stream, ctx(), z);
    if (int rc = launched()) { shmem_free(t->alloc); delete t; return rc; }
    sync_words_add(z);
    *team_out = t;
    return SHMEM_OK;
}

int shmem_team_destroy(shmem_team_t t)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!t) return SHMEM_ERR_INVALID_ARG;
    sync_words_remove(shmemx::GinState{t->st.words_off, t->st.words_off, 32u, 0u});
    int rc = shmem_free(t->alloc);
    delete t;
    return rc;
}

int shmem_team_device_state(shmem_team_t t, shmem_pe_team *state_out)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!t || !state_out) return SHMEM_ERR_INVALID_ARG;
    memcpy(state_out, &t->st, sizeof t->st);
    return SHMEM_OK;
}

int shmem_team_sync(shmem_team_t t, int wgs_per_pe)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!t || !grid_fits(wgs_per_pe)) return SHMEM_ERR_INVALID_ARG;
    long grid = (long)H.npes * wgs_per_pe;
    if (grid > max_resident_wgs(shmemx::k_team_sync)) return SHMEM_ERR_INVALID_ARG;
    shmemx::Ctx c = ctx();
    shmemx::PeTeam st = t->st;
    uint32_t w = (uint32_t)wgs_per_pe;
    void *args[] = {&c, &st, &w};
    return launch_resident((const void *)shmemx::k_team_sync, dim3((unsigned)grid), dim3(WG_THREADS), args);
}

int shmem_team_epochs(const shmem_team_t *teams, const int *rounds, int nteams, uint64_t *slots_sym, int wgs_per_pe,
                      uint64_t *dev_errors)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (nteams < 0 || nteams > (int)shmemx::TEAM_EPOCHS_MAX || (nteams && (!teams || !rounds)) || !grid_fits(wgs_per_pe)) return SHMEM_ERR_INVALID_ARG;
    if ((uintptr_t)slots_sym % 8 || (uintptr_t)dev_errors % 8) return SHMEM_ERR_ALIGN;
    uint64_t off;
    if (int rc = sym_off(slots_sym, 8ull * (uint64_t)H.npes, &off)) return rc;
    shmemx::TeamEpochsArgs a;
    memset(&a, 0, sizeof a);
    std::vector<char> taken((size_t)H.npes, 0);
    bool work = false;
    for (int k = 0; k < nteams; ++k) {
        if (!teams[k] || rounds[k] < 0) return SHMEM_ERR_INVALID_ARG;
        a.team[k] = teams[k]->st;
        a.rounds[k] = (uint32_t)rounds[k];
        work |= rounds[k] > 0;
        for (uint32_t i = 0; i < a.team[k].size; ++i) {                  // a PE runs the rounds of ONE team
            char &seen = taken[a.team[k].start + i * a.team[k].stride];
            if (seen) return SHMEM_ERR_INVALID_ARG;
            seen = 1;
        }
    }
    if (!work) return SHMEM_OK;
    long grid = (long)H.npes * wgs_per_pe;
    if (grid > max_resident_wgs(shmemx::k_team_epochs)) return SHMEM_ERR_INVALID_ARG;
    a.nteams = (uint32_t)nteams; a.wgs_per_pe = (uint32_t)wgs_per_pe; a.slots_off = off; a.errors = dev_errors;
    shmemx::Ctx c = ctx();
    void *args[] = {&c, &a};
    return launch_resident((const void *)shmemx::k_team_epochs, dim3((unsigned)grid), dim3(WG_THREADS), args);
}

int shmem_fence_litmus(void *buf_sym, size_t nbytes, int rounds, int use_quiet, uint64_t *dev_errors)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (H.npes < 2 || rounds < 0 || nbytes % 8) return SHMEM_ERR_INVALID_ARG;
    if ((uintptr_t)buf_sym % 8 || (uintptr_t)dev_errors % 8) return SHMEM_ERR_ALIGN;
    if (nbytes > H.seg) return SHMEM_ERR_OUT_OF_RANGE;
    const uint64_t span = ((uint64_t)nbytes + 255) / 256 * 256 + 512;
    uint64_t boff;
    if (int rc = sym_off(buf_sym, span, &boff)) return rc;
    if (rounds == 0) return SHMEM_OK;
    if (2 > max_resident_wgs(shmemx::k_fence_litmus)) return SHMEM_ERR_DEVICE;
    shmemx::Ctx c = ctx();
    uint64_t nb = nbytes;
    uint32_t r = (uint32_t)rounds;
    void *args[] = {&c, &boff, &nb, &r, &use_quiet, &dev_errors};
    return launch_resident((const void *)shmemx::k_fence_litmus, dim3(2), dim3(WG_THREADS), args);
}

// ---------------------------------------------------------------------------
struct shmem_moe {
    shmemx::MoeState st;
    void *recv_alloc, *comb_alloc, *sig_alloc;   // no call counters here: a launch replayed from a graph must find all its state on the device
};

int shmem_moe_create(int num_experts, int max_tokens, int topk, size_t hidden_bytes, shmem_moe_t *moe_out)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!moe_out || num_experts < 1 || max_tokens < 1 || topk < 1 || hidden_bytes == 0) return SHMEM_ERR_INVALID_ARG;
    if (num_experts % H.npes || (uint32_t)num_experts > shmemx::MOE_MAX_EXPERTS || (uint32_t)max_tokens > shmemx::MOE_MAX_TOKENS ||
        (uint32_t)topk > shmemx::MOE_MAX_TOPK || topk > num_experts || (uint32_t)H.npes > shmemx::MOE_MAX_PES ||
        hidden_bytes % 16 || hidden_bytes > (1u << 30)) return SHMEM_ERR_INVALID_ARG;
    shmem_moe *m = new (std::nothrow) shmem_moe();
    if (!m) return SHMEM_ERR_NOMEM;
    shmemx::MoeState &st = m->st;
    st.num_experts = (uint32_t)num_experts; st.epp = (uint32_t)(num_experts / H.npes);
    st.max_tokens = (uint32_t)max_tokens; st.topk = (uint32_t)topk;
    st.hidden = hidden_bytes; st.msg = hidden_bytes + shmemx::MOE_META_BYTES;
    const uint32_t nsig = st.epp * (uint32_t)H.npes + st.num_experts + shmemx::MOE_CTL_WORDS;   // dispatch counts, combine flags, the PE's control words
    unsigned __int128 recv_bytes = (unsigned __int128)st.epp * (unsigned)H.npes * (unsigned)max_tokens * st.msg;
    unsigned __int128 comb_bytes = (unsigned __int128)max_tokens * (unsigned)topk * st.hidden;
    if (recv_bytes > H.seg || comb_bytes > H.seg) { delete m; return SHMEM_ERR_NOMEM; }
    m->recv_alloc = shmem_malloc((size_t)recv_bytes);
    m->comb_alloc = m->recv_alloc ? shmem_malloc((size_t)comb_bytes) : nullptr;
    m->sig_alloc = m->comb_alloc ? shmem_malloc((size_t)nsig * 8) : nullptr;
    if (!m->sig_alloc) {
        if (m->comb_alloc) shmem_free(m->comb_alloc);
        if (m->recv_alloc) shmem_free(m->recv_alloc);
        delete m;
        return SHMEM_ERR_NOMEM;
    }
    st.recv_off = (uint64_t)((uint8_t *)m->recv_alloc - H.heap);
    st.comb_off = (uint64_t)((uint8_t *)m->comb_alloc - H.heap);
    st.gin.signals_off = (uint64_t)((uint8_t *)m->sig_alloc - H.heap);
    st.gin.counters_off = st.gin.signals_off;
    st.gin.nsignals = nsig; st.gin.ncounters = 0;
    hipLaunchKernelGGL(shmemx::k_gin_zero, dim3((unsigned)std::min(H.npes, 1024)), dim3(256), 0, H.stream, ctx(), st.gin);
    if (int rc = launched()) { shmem_moe_destroy(m); return rc; }
    sync_words_add(st.gin);
    *moe_out = m;
    return SHMEM_OK;
}

int shmem_moe_destroy(shmem_moe_t m)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!m) return SHMEM_ERR_INVALID_ARG;
    sync_words_remove(m->st.gin);
    int rc = shmem_free(m->sig_alloc);
    int rc2 = shmem_free(m->comb_alloc);
    int rc3 = shmem_free(m->recv_alloc);
    delete m;
    return rc ? rc : rc2 ? rc2 : rc3;
}

int shmem_moe_dispatch(shmem_moe_t m, const void *dev_x, const int32_t *dev_topk, const int32_t *dev_ntok,
                       void *dev_recv_x, int32_t *dev_recv_info, int32_t *dev_recv_range, int32_t *dev_recv_count,
                       int wgs_per_pe)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!m || !dev_x || !dev_topk || !dev_ntok || !dev_recv_x || !dev_recv_info || !dev_recv_range || !dev_recv_count ||
        !grid_fits(wgs_per_pe)) return SHMEM_ERR_INVALID_ARG;
    if (((uintptr_t)dev_x | (uintptr_t)dev_recv_x | (uintptr_t)dev_recv_info | (uintptr_t)dev_topk) % 16) return SHMEM_ERR_ALIGN;
    long grid = (long)H.npes * wgs_per_pe;
    if (grid > max_resident_wgs(shmemx::k_moe_dispatch, shmemx::MOE_THREADS)) return SHMEM_ERR_INVALID_ARG;
    shmemx::Ctx c = ctx();
    shmemx::MoeState st = m->st;
    shmemx::MoeDispatchArgs a{(const uint8_t *)dev_x, dev_topk, dev_ntok, (uint8_t *)dev_recv_x, dev_recv_info,
                              dev_recv_range, dev_recv_count, (uint32_t)wgs_per_pe};
    void *args[] = {&c, &st, &a};
    return launch_resident((const void *)shmemx::k_moe_dispatch, dim3((unsigned)grid), dim3(shmemx::MOE_THREADS), args);
}

int shmem_moe_combine(shmem_moe_t m, const void *dev_expert_out, const int32_t *dev_recv_info,
                      const int32_t *dev_recv_range, const int32_t *dev_topk, const int32_t *dev_ntok,
                      void *dev_combined, int wgs_per_pe)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!m || !dev_expert_out || !dev_recv_info || !dev_recv_range || !dev_topk || !dev_ntok || !dev_combined ||
        !grid_fits(wgs_per_pe)) return SHMEM_ERR_INVALID_ARG;
    if (((uintptr_t)dev_expert_out | (uintptr_t)dev_combined | (uintptr_t)dev_recv_info) % 16) return SHMEM_ERR_ALIGN;
    long grid = (long)H.npes * wgs_per_pe;
    if (grid > max_resident_wgs(shmemx::k_moe_combine, shmemx::MOE_THREADS)) return SHMEM_ERR_INVALID_ARG;
    shmemx::Ctx c = ctx();
    shmemx::MoeState st = m->st;
    shmemx::MoeCombineArgs a{(const uint8_t *)dev_expert_out, dev_recv_info, dev_recv_range, dev_topk, dev_ntok,
                             (uint8_t *)dev_combined, (uint32_t)wgs_per_pe};
    void *args[] = {&c, &st, &a};
    return launch_resident((const void *)shmemx::k_moe_combine, dim3((unsigned)grid), dim3(shmemx::MOE_THREADS), args);
}

// ---------------------------------------------------------------------------
// Proxy-style executor (Sec. III-C, "Proxy Backend"): the host half.  One thread per proxy object
// polls the descriptor ring in pinned memory, takes descriptors out in ticket order, validates them
// on the host and carries them out on a stream of its own: contiguous ops through the copy engine
// (hipMemcpyAsync), strided ops with the library's strided kernel.  `head` (GPU-visible) tells the
// producers which slots are free again; `executed` counts descriptors handed to the stream.
struct shmem_proxy {
    shmemx::ProxyQueue q;
    uint64_t entries;
    uint64_t *head;                     // pinned, written by the thread, read by the GPU
    hipStream_t stream;
    hipEvent_t ready;                   // orders the proxy stream behind the library's stream at submit
    int device;
    std::thread worker;
    std::atomic<bool> stop{false};
    std::atomic<uint64_t> executed{0};  // descriptors taken out and handed to the stream
    std::atomic<uint64_t> rejected{0};
    std::atomic<uint64_t> first_bad{UINT64_MAX};
    std::atomic<int> hip_error{0};
    uint64_t submitted = 0;             // descriptors given to shmem_proxy_submit so far (caller's thread)
    // captured at creation: the heap the descriptors refer to
    uint8_t *heap; uint64_t seg; int npes;
};

namespace {

bool proxy_desc_valid(const shmem_proxy *p, const shmem_op_desc &d)
{
    return hostlogic::desc_valid(d, (uint32_t)p->npes, p->seg);
}

void proxy_execute(shmem_proxy *p, const shmem_op_desc &d)
{
    uint8_t *local = p->heap + (uint64_t)d.pe_self * p->seg + d.local_off;
    uint8_t *remote = p->heap + (uint64_t)d.pe * p->seg + d.sym_off;
    hipError_t e = hipSuccess;
    if (d.count == 0) return;
    switch (d.kind) {
    case SHMEM_OP_PUT: e = hipMemcpyAsync(remote, local, d.count, hipMemcpyDeviceToDevice, p->stream); break;
    case SHMEM_OP_GET: e = hipMemcpyAsync(local, remote, d.count, hipMemcpyDeviceToDevice, p->stream); break;
    case SHMEM_OP_IPUT:
        hipLaunchKernelGGL(shmemx::k_strided, dim3(wgs_for_bytes(d.count * 16)), dim3(WG_THREADS), 0, p->stream, remote,
                           (const uint8_t *)local, d.sym_stride, d.local_stride, (size_t)d.count, d.elem_bytes);
        e = hipGetLastError();
        break;
    case SHMEM_OP_IGET:
        hipLaunchKernelGGL(shmemx::k_strided, dim3(wgs_for_bytes(d.count * 16)), dim3(WG_THREADS), 0, p->stream, local,
                           (const uint8_t *)remote, d.local_stride, d.sym_stride, (size_t)d.count, d.elem_bytes);
        e = hipGetLastError();
        break;
    }
    if (e != hipSuccess) p->hip_error.store((int)e);
}

void proxy_main(shmem_proxy *p)
{
    if (hipSetDevice(p->device) != hipSuccess) { p->hip_error.store(1); return; }
    uint64_t next = 0, idle = 0;
    while (!p->stop.load(std::memory_order_acquire)) {
        const uint64_t slot = next & p->q.mask;
        if (__atomic_load_n(p->q.flags + slot, __ATOMIC_ACQUIRE) != next + 1) {
            if (++idle > 2000) std::this_thread::sleep_for(std::chrono::microseconds(20));   // nothing for a while
            continue;
        }
        idle = 0;
        const shmem_op_desc d = p->q.ring[slot];                 // take the descriptor out ...
        __atomic_store_n(p->head, next + 1, __ATOMIC_RELEASE);   // ... and hand the slot back to the producers
        if (proxy_desc_valid(p, d)) {
            proxy_execute(p, d);
        } else {
            p->rejected.fetch_add(1);
            uint64_t expect = UINT64_MAX;
            p->first_bad.compare_exchange_strong(expect, next);
        }
        ++next;
        p->executed.store(next, std::memory_order_release);
    }
}

void proxy_stop_and_free(shmem_proxy *p)
{
    p->stop.store(true, std::memory_order_release);
    if (p->worker.joinable()) p->worker.join();
    (void)hipStreamSynchronize(p->stream);
    (void)hipEventDestroy(p->ready);
    (void)hipStreamDestroy(p->stream);
    (void)hipHostFree(p->q.ring);
    (void)hipHostFree(p->q.flags);
    (void)hipHostFree(p->head);
    H.proxies.erase(std::remove(H.proxies.begin(), H.proxies.end(), p), H.proxies.end());
    delete p;
}

}  // namespace

int shmem_proxy_create(size_t queue_entries, shmem_proxy_t *proxy_out)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!proxy_out || queue_entries < 2 || queue_entries > (1u << 20) || (queue_entries & (queue_entries - 1)))
        return SHMEM_ERR_INVALID_ARG;
    shmem_proxy *p = new (std::nothrow) shmem_proxy();
    if (!p) return SHMEM_ERR_NOMEM;
    p->entries = queue_entries;
    p->heap = H.heap; p->seg = H.seg; p->npes = H.npes;
    void *ring = nullptr, *flags = nullptr, *head = nullptr;
    const unsigned fl = hipHostMallocMapped | hipHostMallocCoherent;
    bool ok = hipGetDevice(&p->device) == hipSuccess &&
              hipHostMalloc(&ring, queue_entries * sizeof(shmem_op_desc), fl) == hipSuccess &&
              hipHostMalloc(&flags, queue_entries * sizeof(uint64_t), fl) == hipSuccess &&
              hipHostMalloc(&head, 256, fl) == hipSuccess &&
              hipStreamCreateWithFlags(&p->stream, hipStreamNonBlocking) == hipSuccess;
    if (ok && hipEventCreateWithFlags(&p->ready, hipEventDisableTiming) != hipSuccess) { (void)hipStreamDestroy(p->stream); ok = false; }
    if (!ok) {
        if (ring) (void)hipHostFree(ring);
        if (flags) (void)hipHostFree(flags);
        if (head) (void)hipHostFree(head);
        delete p;
        return SHMEM_ERR_DEVICE;
    }
    memset(ring, 0, queue_entries * sizeof(shmem_op_desc));
    memset(flags, 0, queue_entries * sizeof(uint64_t));
    memset(head, 0, 256);
    p->q.ring = (shmem_op_desc *)ring; p->q.flags = (uint64_t *)flags; p->q.head = (const uint64_t *)head;
    p->q.mask = queue_entries - 1;
    p->head = (uint64_t *)head;
    p->worker = std::thread(proxy_main, p);
    {
        std::lock_guard<std::mutex> g(H.mu);
        H.proxies.push_back(p);
    }
    *proxy_out = p;
    return SHMEM_OK;
}

int shmem_proxy_submit(shmem_proxy_t p, const void *dev_ops, size_t n, int workgroups)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!p || (!dev_ops && n) || workgroups < 1) return SHMEM_ERR_INVALID_ARG;
    if ((uintptr_t)dev_ops % 16) return SHMEM_ERR_ALIGN;
    if (n == 0) return SHMEM_OK;
    // every producer must be resident: a waiting producer of a high ticket must not keep a low one off the device
    if (workgroups > max_resident_wgs(shmemx::k_proxy_submit)) return SHMEM_ERR_INVALID_ARG;
    // what the library's stream has done so far happens before the proxy's copies of this submission
    if (hipEventRecord(p->ready, H.stream) != hipSuccess || hipStreamWaitEvent(p->stream, p->ready, 0) != hipSuccess)
        return SHMEM_ERR_DEVICE;
    hipLaunchKernelGGL(shmemx::k_proxy_submit, dim3((unsigned)workgroups), dim3(WG_THREADS), 0, H.stream, ctx(), p->q,
                       (const shmem_op_desc *)dev_ops, (uint64_t)n, p->submitted);
    if (int rc = launched()) return rc;
    p->submitted += n;
    return SHMEM_OK;
}

int shmem_proxy_quiet(shmem_proxy_t p, uint64_t *first_bad_index)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!p) return SHMEM_ERR_INVALID_ARG;
    const auto t0 = std::chrono::steady_clock::now();
    while (p->executed.load(std::memory_order_acquire) < p->submitted) {
        if (p->hip_error.load()) return SHMEM_ERR_DEVICE;
        if (std::chrono::steady_clock::now() - t0 > std::chrono::seconds(20)) return SHMEM_ERR_DEVICE;   // a producer gave up
        std::this_thread::yield();
    }
    if (hipStreamSynchronize(p->stream) != hipSuccess || p->hip_error.load()) return SHMEM_ERR_DEVICE;
    if (p->rejected.load()) {
        if (first_bad_index) *first_bad_index = p->first_bad.load();
        return SHMEM_ERR_DEVICE_FAULT;
    }
    return SHMEM_OK;
}

int shmem_proxy_stats(shmem_proxy_t p, uint64_t *submitted, uint64_t *executed, uint64_t *rejected)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!p) return SHMEM_ERR_INVALID_ARG;
    if (submitted) *submitted = p->submitted;
    if (executed) *executed = p->executed.load();
    if (rejected) *rejected = p->rejected.load();
    return SHMEM_OK;
}

int shmem_proxy_destroy(shmem_proxy_t p)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    (void)hipStreamSynchronize(H.stream);            // no producer is still writing into the ring
    std::lock_guard<std::mutex> g(H.mu);
    if (!p || std::find(H.proxies.begin(), H.proxies.end(), p) == H.proxies.end()) return SHMEM_ERR_INVALID_ARG;
    proxy_stop_and_free(p);
    return SHMEM_OK;
}

// ---------------------------------------------------------------------------
int shmem_transpose(void *out_sym, const void *in_sym, size_t n, size_t elem_bytes, int wgs_per_pe)
{
    if (!H.init) return SHMEM_ERR_NOT_INIT;
    if (!grid_fits(wgs_per_pe) || (elem_bytes != 4 && elem_bytes != 8)) return SHMEM_ERR_INVALID_ARG;
    if (n % (size_t)H.npes) return SHMEM_ERR_INVALID_ARG;
    if (((uintptr_t)out_sym | (uintptr_t)in_sym) % elem_bytes) return SHMEM_ERR_ALIGN;
    const size_t rows = n / (size_t)H.npes;
    unsigned __int128 span = (unsigned __int128)rows * n * elem_bytes;
    if (span > H.seg) return SHMEM_ERR_OUT_OF_RANGE;
    uint64_t ooff, ioff;
    if (int rc = sym_off(out_sym, (uint64_t)span, &ooff)) return rc;
    if (int rc = sym_off(in_sym, (uint64_t)span, &ioff)) return rc;
    if (span && ooff < ioff + (uint64_t)span && ioff < ooff + (uint64_t)span) return SHMEM_ERR_INVALID_ARG;   // not in place
    if (n == 0) return SHMEM_OK;
    shmemx::TransposeArgs a{ioff, ooff, (uint64_t)n, (uint64_t)rows, (uint32_t)wgs_per_pe};
    dim3 grid((unsigned)(H.npes * wgs_per_pe)), block(WG_THREADS);
    const size_t vec_elems = 16 / elem_bytes;
    const bool wide = rows % vec_elems == 0 && ((ooff | ioff) & 15) == 0;   // then n % vec_elems == 0, too
    if (elem_bytes == 4) {
        if (wide) hipLaunchKernelGGL((shmemx::k_transpose_vec<uint32_t, 128>), grid, block, 0, H.stream, ctx(), a);
        else hipLaunchKernelGGL(shmemx::k_transpose<uint32_t>, grid, block, 0, H.stream, ctx(), a);
    } else {
        if (wide) hipLaunchKernelGGL((shmemx::k_transpose_vec<uint64_t, 64>), grid, block, 0, H.stream, ctx(), a);
        else hipLaunchKernelGGL(shmemx::k_transpose<uint64_t>, grid, block, 0, H.stream, ctx(), a);
    }
    return launched();
}

}  // extern "C"

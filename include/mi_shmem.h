/*
 * mi_shmem -- one-sided (PGAS / OpenSHMEM-style) communication primitives on a
 * single MI355X, with processing elements (PEs) emulated as workgroup teams
 * that share one symmetric heap in HBM.
 *
 * C ABI.  Every pointer argument says whether it is a HOST or a DEVICE pointer.
 * Nothing here allocates device memory: the caller owns the heap, the scratch
 * words, every dev_* array and the HIP stream, and keeps them alive until
 * shmem_finalize().  The library owns only host-side allocator metadata.
 *
 * Model
 *   - shmem_init() is given one device buffer of npes * heap_bytes_per_pe
 *     bytes.  PE p's segment is [p * heap_bytes_per_pe, (p+1) * heap_bytes_per_pe).
 *     Buffers are registered from an existing allocation; allocation and
 *     registration are decoupled and every segment has the same size
 *     (Sec. III-A, "Windows-based symmetric memory").
 *   - A SYMMETRIC ADDRESS is a device address inside PE 0's segment (what
 *     shmem_malloc returns).  Together with a PE number it names that PE's copy:
 *     shmem_ptr(sym, pe) = sym + pe * heap_bytes_per_pe.
 *   - A LOCAL address is an ordinary device pointer (for the initiator's own
 *     copy of a symmetric object pass shmem_ptr(sym, pe_self)).
 *   - Every call that moves data is STREAM-ORDERED on the stream given to
 *     shmem_init and executed entirely by device kernels; pe_self names the
 *     emulated initiator, whose workgroup team performs the operation.
 *
 * Status: 0 = OK, < 0 = error.  Errors that the host can see (not initialised,
 * bad PE, address outside a segment, range overrun, stride < 1, misalignment,
 * heap exhausted) are returned at once and enqueue nothing.  Errors only the
 * device can see (a bad descriptor inside a device-resident table) set a
 * device error word, skip that op and surface at shmem_stream_sync().
 * No exceptions, no abort(), nothing printed.  Every wgs_per_pe argument must
 * be at least 1 and npes * wgs_per_pe at most 2^22 (INVALID_ARG otherwise).
 *
 * The library keeps ONE context per process (init ... finalize).  The allocator
 * calls take a lock; everything else expects one calling thread at a time.
 * All entry points are stream-ordered except shmem_bfs, shmem_stream_sync,
 * shmem_init and shmem_finalize, which block the host.  The stream-ordered ones
 * only launch kernels and keep no per-call state on the host, so they may be
 * captured into a HIP graph and replayed (not: the proxy calls, which involve
 * a host thread, and the create / destroy calls).
 */
#ifndef MI_SHMEM_H
#define MI_SHMEM_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    SHMEM_OK = 0,
    SHMEM_ERR_NOT_INIT = -1,
    SHMEM_ERR_ALREADY_INIT = -2,
    SHMEM_ERR_INVALID_ARG = -3,
    SHMEM_ERR_INVALID_PE = -4,
    SHMEM_ERR_OUT_OF_RANGE = -5,
    SHMEM_ERR_ALIGN = -6,
    SHMEM_ERR_NOMEM = -7,
    SHMEM_ERR_BAD_FREE = -8,
    SHMEM_ERR_DEVICE = -9,       /* a HIP runtime call failed            */
    SHMEM_ERR_DEVICE_FAULT = -10 /* an op was rejected on the device     */
};
/* HOST: static string for a status code. */
const char *shmem_strerror(int status);

/* ---- set-up (Sec. III-B "Usage workflow": create, register, use) ---------- */

/* Bytes of zero-initialisable device scratch the library needs for npes PEs
 * (barrier words, device error word, work counters).  0 if npes < 1. */
size_t shmem_scratch_bytes(int npes);

/* dev_heap: DEVICE, npes * heap_bytes_per_pe bytes, 256-byte aligned;
 * heap_bytes_per_pe a multiple of 256.  dev_scratch: DEVICE,
 * shmem_scratch_bytes(npes) bytes, 256-byte aligned; the library zeroes it.
 * hip_stream: a hipStream_t (NULL = the default stream).
 * Both buffers must come from the HIP runtime this library is linked to: a
 * process that holds a second copy of the runtime (a Python wheel that ships
 * its own) loads that one FIRST, so that the library binds to it, or the
 * pointers mean nothing here (DEVICE).  If the runtime can name the
 * allocation behind a buffer and it is shorter than stated: OUT_OF_RANGE.
 * Errors: ALREADY_INIT, INVALID_ARG, ALIGN, OUT_OF_RANGE, DEVICE. */
int shmem_init(int npes, size_t heap_bytes_per_pe, void *dev_heap, void *dev_scratch, void *hip_stream);
/* Waits for the stream, forgets everything.  Live allocations are dropped. */
int shmem_finalize(void);
int shmem_n_pes(void);                 /* 0 when not initialised */

/* Symmetric allocator (same offset on every PE).  Address-ordered first fit,
 * 256-byte granularity and minimum alignment, neighbours coalesced on free.
 * Return a symmetric address (DEVICE, inside PE 0's segment) or NULL on
 * failure / nbytes == 0 / alignment not a power of two.  Host-side only. */
void *shmem_malloc(size_t nbytes);
void *shmem_align(size_t alignment, size_t nbytes);
int shmem_free(void *sym);             /* BAD_FREE unless sym came from malloc/align */
/* Address of PE pe's copy; NULL if sym is not inside PE 0's segment or pe is
 * out of range. */
void *shmem_ptr(const void *sym, int pe);

/* ---- one-sided data movement (Sec. III-A; Table II put / get) ------------- */
/* Errors of the five calls below: NOT_INIT; INVALID_PE (pe_self or pe);
 * OUT_OF_RANGE (the symmetric range leaves the segment, or a stride / count
 * overflows); INVALID_ARG (a NULL local pointer with bytes to move, a stride
 * < 1, an element size other than 1, 2, 4, 8); ALIGN (iput / iget addresses,
 * the signal word); DEVICE.  The local side is an ordinary device pointer and
 * is NOT range-checked: the caller owns it. */

/* put: copy nbytes from src_local (DEVICE) to PE pe's copy of dst_sym.  The
 * source is reusable once the call is stream-complete; delivery is guaranteed
 * after shmem_quiet / shmem_barrier_all (here: by stream order).  nbytes == 0
 * and pe == pe_self are legal.  Source and destination must not overlap. */
int shmem_put(int pe_self, void *dst_sym, const void *src_local, size_t nbytes, int pe);
/* get: copy nbytes from PE pe's copy of src_sym to dst_local (DEVICE); blocking
 * in stream order. */
int shmem_get(int pe_self, void *dst_local, const void *src_sym, size_t nbytes, int pe);
/* put with a signal: the put above, then `value` is added to PE pe's copy of
 * sig_sym (symmetric uint64, 8-byte aligned) and lands only after the data is
 * visible there -- the paper's put with the SignalAdd{value} action (SignalInc:
 * value 1; Sec. III-A "Ordering semantics"), OpenSHMEM's put_signal with
 * SIGNAL_ADD.  nbytes == 0 is the zero-byte put + signal that the paper uses
 * as a release.  Both halves are checked before either is enqueued. */
int shmem_put_signal(int pe_self, void *dst_sym, const void *src_local, size_t nbytes, uint64_t *sig_sym,
                     uint64_t value, int pe);
/* iput: dest[i * dst_stride] = src[i * src_stride] for i < nelems; strides in
 * elements, >= 1; elem_bytes in {1,2,4,8}; both addresses aligned to it.
 * Bytes between destination elements are not written. */
int shmem_iput(int pe_self, void *dst_sym, const void *src_local, ptrdiff_t dst_stride,
               ptrdiff_t src_stride, size_t nelems, size_t elem_bytes, int pe);
/* iget: the mirror of iput (strided read from PE pe, strided local write). */
int shmem_iget(int pe_self, void *dst_local, const void *src_sym, ptrdiff_t dst_stride,
               ptrdiff_t src_stride, size_t nelems, size_t elem_bytes, int pe);

/* ---- atomic memory operations on a 64-bit word (Table II memory atomics) -- */
/* Each is indivisible with respect to every other AMO on the same word and
 * writes the previous value to *dev_result (DEVICE, may be NULL).  dst_sym:
 * symmetric, 8-byte aligned.  compare_swap stores `value` if the word equals
 * `cond`.  Errors: NOT_INIT, INVALID_PE, OUT_OF_RANGE, ALIGN, DEVICE. */
int shmem_atomic_fetch_add(int pe_self, uint64_t *dst_sym, uint64_t value, int pe, uint64_t *dev_result);
int shmem_atomic_compare_swap(int pe_self, uint64_t *dst_sym, uint64_t cond, uint64_t value, int pe,
                              uint64_t *dev_result);
int shmem_atomic_fetch_or(int pe_self, uint64_t *dst_sym, uint64_t value, int pe, uint64_t *dev_result);

/* ---- ordering (Sec. III-A "Ordering semantics"; Table II quiet / barrier) - */
/* fence: earlier puts of pe_self to a PE are delivered before its later puts
 * to that PE.  quiet: earlier puts and AMOs of pe_self (-1: of every PE) are
 * complete and visible to all PEs -- the stronger reading, unlike the paper's
 * flush, which only promises that sources are reusable.  barrier_all: quiet
 * on every PE, then all PEs synchronise.  At this host level each earlier call
 * is a finished kernel in stream order, so these enqueue no work; their
 * in-kernel forms are what the batched entry points below execute. */
int shmem_fence(int pe_self);
int shmem_quiet(int pe_self);
int shmem_barrier_all(void);
/* HOST waits for the stream.  DEVICE_FAULT if the device error word is set
 * (the word is then cleared); *first_bad_index (HOST, may be NULL) receives
 * the index of the first rejected op.  If the fault was a bounded wait that
 * gave up (a barrier or signal wait that timed out: some workgroup never
 * arrived), arrival counts and generations are left half-advanced, so the
 * call also starts all synchronisation state afresh before it returns: the
 * scratch words, and the signals, counters and barrier words of every live
 * Gin, team and MoE object read 0 again.  The library is usable as after
 * shmem_init; data in the heap is as the failed launch left it. */
int shmem_stream_sync(uint64_t *first_bad_index);

/* ---- batched entry points: inputs device-resident, one launch each -------- */

/* 64-byte operation descriptor (the record shape of the Proxy backend's
 * queue entries, Sec. III-C: window offsets, sizes, an inline value). */
typedef struct {
    uint32_t kind;        /* SHMEM_OP_*                                        */
    uint32_t pe_self;     /* initiator                                         */
    uint32_t pe;          /* remote PE                                         */
    uint32_t elem_bytes;  /* IPUT/IGET: 1,2,4,8; PUT/GET: ignored              */
    uint64_t local_off;   /* byte offset in the initiator's segment            */
    uint64_t sym_off;     /* byte offset in PE pe's segment                    */
    uint64_t count;       /* PUT/GET: bytes; IPUT/IGET: elements               */
    int64_t local_stride; /* in elements (IPUT/IGET)                           */
    int64_t sym_stride;   /* in elements (IPUT/IGET)                           */
    uint64_t value;       /* reserved for inline-value ops                     */
} shmem_op_desc;
enum { SHMEM_OP_PUT = 0, SHMEM_OP_GET = 1, SHMEM_OP_IPUT = 2, SHMEM_OP_IGET = 3 };

/* Executes n descriptors (DEVICE table) in ONE persistent launch of
 * npes * wgs_per_pe workgroups.  PE team p executes the descriptors whose
 * pe_self is p.  After every quiet_every descriptors (by table index; 0 = only
 * at the end) and at the end every wave performs quiet and all teams meet in
 * an in-kernel world barrier.  Ops between two barriers run concurrently and
 * unordered (GIN operations are unordered by default): a table in which an op
 * writes bytes that another op of the same window reads or writes has no
 * defined result.  A descriptor with a bad kind / PE / range / stride /
 * alignment is skipped and recorded in the device error word.
 * Errors: NOT_INIT, INVALID_ARG (wgs_per_pe < 1 or more workgroups than can be
 * co-resident), DEVICE. */
int shmem_op_batch(const void *dev_ops, size_t n, size_t quiet_every, int wgs_per_pe);

/* The executor above for callers that cannot allocate or register anything:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  It needs no shmem_init and no scratch buffer from the caller: the
 * barrier and fault words it uses are a fixed array inside the library's code
 * object (33,280 bytes, held by every GPU that loads the library until the
 * process ends), which limits it to npes <= 64 (OUT_OF_RANGE beyond).  The
 * call allocates and frees nothing; it launches kernels on hip_stream only (a
 * fill of the words it uses, the executor, and -- if dev_fault is given -- a
 * copy of the fault words) and is asynchronous.
 * dev_heap: DEVICE, npes * heap_bytes_per_pe bytes, 256-byte aligned, segment
 * size a multiple of 256; dev_ops: DEVICE table of n descriptors whose offsets
 * refer to that heap; dev_fault: DEVICE uint64[2] (may be NULL) that receives
 * the device error word and the index of the first rejected descriptor (0, 0 =
 * none) once the stream has reached that point.  Same table semantics, same
 * heap contents afterwards as shmem_op_batch.  All calls on one GPU share the
 * one array: calls that overlap in time on a GPU (two streams, two threads)
 * race on the barrier words and must be serialised by the caller.
 * Errors: INVALID_ARG (also: more workgroups than can be co-resident),
 * OUT_OF_RANGE (npes > 64), ALIGN, DEVICE. */
int shmem_op_batch_noalloc(int npes, size_t heap_bytes_per_pe, void *dev_heap, const void *dev_ops, size_t n,
                           size_t quiet_every, int wgs_per_pe, uint64_t *dev_fault, void *hip_stream);

/* Bandwidth sweep cell.  Every PE p, as initiator, issues ops_per_pe operations
 * of `kind` towards PE (p+1) mod npes, back to back in one launch of at most
 * npes * wgs_per_pe workgroups.  Op k works on slot k mod nslots: the local
 * buffer at local_sym + slot * local_slot_bytes in p's own segment and the
 * remote buffer at remote_sym + slot * remote_slot_bytes in the peer's segment.
 * PUT/GET move `count` bytes; IPUT/IGET move `count` elements of elem_bytes
 * with the given strides (local_stride applies to the local side).  The ops of
 * a cell are independent and unordered; completion is the kernel boundary.
 * Bandwidth cells -- PUT/GET of 256 bytes and more with 16-byte aligned sizes and
 * placement, asked for with at least one workgroup per compute unit -- run on
 * one larger workgroup per compute unit (compute units / npes per PE) that
 * streams through LDS at a paced rate.  Where a PE's operations make enough
 * work (whole multiples of 4 KiB: at least 32 tasks of 4 KiB per workgroup in
 * whole blocks of four; other sizes: messages that fill at least nine tenths
 * of their 1 KiB rows, at least 128 rows per workgroup; messages of 512 bytes,
 * and of 256 bytes when fewer than 128 workgroups per PE are asked for, two or
 * four to a row, if ops_per_pe and nslots are multiples of that and the rows are
 * as many) the workgroups claim
 * it block by block from a per-PE counter in the scratch words (the counters
 * are zero between launches; MI_SHMEM_STREAM_DYNAMIC=0 in the environment of
 * shmem_init switches that off); else whole multiples of 4 KiB walk fixed
 * shares, and everything else takes the register path.
 * shmem_copy_sweep_geometry tells which launch a cell gets.  Errors as for the
 * single ops, checked for the last slot too. */
int shmem_copy_sweep(int kind, void *remote_sym, void *local_sym, size_t count, size_t elem_bytes,
                     ptrdiff_t remote_stride, ptrdiff_t local_stride, size_t remote_slot_bytes,
                     size_t local_slot_bytes, size_t nslots, int ops_per_pe, int wgs_per_pe);
/* HOST: the launch that shmem_copy_sweep makes for a contiguous or strided
 * cell with these arguments: *workgroups_out workgroups of *threads_out
 * threads (either may be NULL).  Enqueues nothing.
 * Errors: NOT_INIT, INVALID_ARG. */
int shmem_copy_sweep_geometry(int kind, void *remote_sym, void *local_sym, size_t count, size_t remote_slot_bytes,
                              size_t local_slot_bytes, size_t nslots, int ops_per_pe, int wgs_per_pe,
                              int *workgroups_out /* HOST */, int *threads_out /* HOST */);

/* n AMOs on the symmetric counter array ctr_sym (uint64[T] on every PE).
 * Op i targets word dev_idx[i] of PE dev_pe[i] and is issued by PE
 * i / ceil(n / npes).  kind FETCH_ADD: add dev_a[i]; COMPARE_SWAP: cond dev_a[i],
 * value dev_b[i]; FETCH_OR: or dev_a[i]; MIN_CAS_LOOP: store dev_a[i] if the
 * word is 0 or larger, through a compare-swap retry loop.  dev_old[i]
 * (DEVICE, may be NULL) receives the fetched value.  All arrays DEVICE.
 * `aggregate` != 0 lets a workgroup combine its ops on the same word before
 * they reach memory (FETCH_ADD, FETCH_OR, MIN_CAS_LOOP); results -- final
 * words and fetched values -- are indistinguishable from some serial order
 * either way (for MIN_CAS_LOOP the fetched value is what the word held just
 * before the op in that order). */
enum { SHMEM_AMO_FETCH_ADD = 0, SHMEM_AMO_COMPARE_SWAP = 1, SHMEM_AMO_FETCH_OR = 2, SHMEM_AMO_MIN_CAS_LOOP = 3 };
int shmem_amo_batch(int kind, uint64_t *ctr_sym, size_t T, const int32_t *dev_pe, const uint32_t *dev_idx,
                    const uint64_t *dev_a, const uint64_t *dev_b, uint64_t *dev_old, size_t n,
                    int wgs_per_pe, int aggregate);

/* Distributed open-addressing hash table: table_sym is uint64[slots_per_pe]
 * on every PE, 0 = empty, keys != 0.  h = mix64(key) (the SplitMix64
 * finaliser); owner = h mod npes; home = (h / npes) mod slots_per_pe; linear
 * probing inside the owner's table.  insert: compare_swap(slot, 0, key) per
 * probe; dev_status[i] (DEVICE, may be NULL) = INSERTED / DUPLICATE / FULL.
 * lookup: 8-byte gets until the key (dev_found[i] = 1) or an empty slot (0).
 * Key i is held by PE i / ceil(n / npes). */
enum { SHMEM_HASH_INSERTED = 0, SHMEM_HASH_DUPLICATE = 1, SHMEM_HASH_FULL = 2 };
int shmem_hash_insert(uint64_t *table_sym, size_t slots_per_pe, const uint64_t *dev_keys, size_t n,
                      uint8_t *dev_status, int wgs_per_pe);
int shmem_hash_lookup(const uint64_t *table_sym, size_t slots_per_pe, const uint64_t *dev_keys, size_t n,
                      uint8_t *dev_found, int wgs_per_pe);

/* Level-synchronous BFS over a 1D vertex partition.  A vertex is claimed with
 * fetch_or on its owner's visited bitmap; the claimer reserves a slot in the
 * owner's next-frontier queue with fetch_add and puts the vertex, its parent
 * and its level there; levels are separated by quiet + barrier_all.
 * The partition: shmem_bfs_create ranks the vertices by degree (largest first,
 * ties by number); the vertex of rank r is local vertex r / npes of PE
 * r mod npes, so every PE owns vpp = ceil(nverts / npes) vertices with an equal
 * share of every degree class.  The search runs on that numbering; roots,
 * levels and parents cross this boundary in the caller's numbering.
 * shmem_bfs_create takes the CSR arrays (DEVICE: row offsets uint64[nverts+1],
 * neighbours uint32[nnz]; they are only read during the call), writes the graph
 * in the library's numbering (every row sorted by its neighbours' degree rank,
 * the best-connected first) into device memory that the library allocates
 * (4 bytes per CSR entry, 8 per row, two 4-byte maps per vertex; freed by
 * shmem_bfs_destroy; the ranking is host work, once per graph; sorting the rows
 * takes as much again plus the sort's workspace while the call lasts, and is
 * left out -- the rows then only grouped into four classes of rank -- if that
 * memory cannot be had, for nnz >= 2^32 - 1, or with MI_SHMEM_BFS_SORT_ROWS=0
 * in the environment of shmem_init) and allocates
 * the per-PE state from the symmetric heap (bitmap, level, parent, two queues, a
 * long-row list and its scan, per-die bitmap copies, frontier and previous-level
 * bitmaps, counters: about 25.4 bytes per owned vertex; parent and level of a
 * vertex are one 8-byte record there, delivered with one put).
 * Errors: NOMEM, INVALID_ARG (also: row offsets that decrease, a neighbour
 * that is not below nverts), DEVICE. */
typedef struct {
    uint32_t nlevels;           /* number of non-empty frontiers               */
    uint64_t reached;           /* vertices with level >= 0                    */
    uint64_t edges_traversed;   /* (sum of degrees of reached vertices) / 2    */
    uint64_t frontier_size[64]; /* vertices per level, the first 64 levels     */
} shmem_bfs_stats;
#define SHMEM_BFS_NONE 0xFFFFFFFFu
int shmem_bfs_create(uint32_t nverts, const uint64_t *dev_row_off, const uint32_t *dev_nbr,
                     int wgs_per_pe, void **graph_out /* HOST */);
int shmem_bfs_destroy(void *graph);
/* Direction of the levels.  TOP_DOWN (the default) is the method as stated above
 * on every level.  DIRECTION_OPTIMIZING switches a level to bottom-up -- every
 * owner scans its own unvisited vertices and looks for a neighbour in the current
 * frontier with one-sided gets of the owners' frontier bitmaps; claim, parent,
 * level and queue entry are then local writes -- when the frontier's row lengths
 * add up to more than 1/alpha of those of the unvisited vertices, and back to
 * top-down when the frontier is below nverts/beta and shrinking (alpha, beta = 0:
 * the defaults, 30 and 24); the root's own level is always expanded top-down (its
 * frontier is one vertex).  BOTTOM_UP forces bottom-up on every level (for
 * tests).  Levels, frontier sizes and counts are the same in every mode; parents
 * may differ (all are valid).  OR-ing SHMEM_BFS_CANONICAL_PARENTS into the mode
 * adds a pass after the search that rewrites every parent to the smallest
 * neighbour one level up (one-sided 4-byte gets of the neighbours' levels): the
 * one tree that does not depend on who claimed a vertex first.
 * Errors: NOT_INIT, INVALID_ARG. */
enum { SHMEM_BFS_TOP_DOWN = 0, SHMEM_BFS_DIRECTION_OPTIMIZING = 1, SHMEM_BFS_BOTTOM_UP = 2,
       SHMEM_BFS_CANONICAL_PARENTS = 0x100 };
int shmem_bfs_configure(void *graph, int mode, int alpha, int beta);
/* Runs one search; blocks the host (one stream sync per level).  dev_level
 * (int32[nverts], -1 = unreached) and dev_parent (uint32[nverts],
 * SHMEM_BFS_NONE = unreached; parent[root] = root) are DEVICE and may be NULL;
 * stats is HOST and may be NULL.  A search may have any number of levels
 * (nlevels counts them all; a histogram beyond the first 64 follows from
 * dev_level).  A top-down level whose frontier holds at least nverts / 64
 * vertices (and at least 1024) is expanded from a queue that the owner has
 * rewritten in vertex order from the bits claimed in the level before (the
 * same entries; MI_SHMEM_BFS_SORT_DIV in the environment of shmem_init sets
 * another divisor, 0 = never).  Errors: INVALID_ARG (root >= nverts), DEVICE. */
int shmem_bfs(void *graph, uint32_t root, int32_t *dev_level, uint32_t *dev_parent, shmem_bfs_stats *stats);

/* HOST: how the last shmem_bfs on this graph spent its time, level by level:
 * us_out[i] (HOST, may be NULL) = microseconds of host clock around level i's
 * launches and its hand-over to the host, bottom_up_out[i] (HOST, may be
 * NULL) = 1 if that level ran bottom-up; the first min(levels, 64, max_levels)
 * levels, their number in *nlevels_out.  A measurement aid: no device work.
 * Errors: NOT_INIT, INVALID_ARG. */
int shmem_bfs_level_times(void *graph, uint32_t *nlevels_out, float *us_out, uint8_t *bottom_up_out, uint32_t max_levels);

/* ---- the paper's device API shape: signals, counters, put with actions (Sec. III-A, III-B) ---- */

/* A Gin object owns `nsignals` signals (symmetric uint64, remotely incremented:
 * remote completion) and `ncounters` counters (uint64 local to each PE: local
 * completion), addressed by integer ID as in Listing 1.  Both arrays are taken
 * from the symmetric heap and cleared on every PE (stream-ordered).  Kernels
 * built into the library use them through the device-side Gin interface
 * (put with SignalInc / SignalAdd / CounterInc actions, putValue, signal, flush,
 * read/wait/reset of signals and counters, barrier session).
 * Errors: NOT_INIT, INVALID_ARG, NOMEM, DEVICE. */
int shmem_gin_create(int nsignals, int ncounters, void **gin_out /* HOST */);
int shmem_gin_destroy(void *gin);
/* Symmetric address of signal / counter `id` (for inspection with shmem_ptr +
 * a device read); NULL if out of range. */
void *shmem_gin_signal_sym(void *gin, int id);
void *shmem_gin_counter_sym(void *gin, int id);

/* For kernels of the caller's own: what a HIP kernel needs to use the device
 * API of include/mi_shmem_device.hpp (Listing 1: put with actions, putValue,
 * signal, read/wait/reset of signals and counters, flush, barrier) on the
 * registered heap.  Both structs are plain values that are passed to a kernel
 * as arguments; they stay valid until shmem_finalize / shmem_gin_destroy.
 * The caller launches such kernels on the stream given to shmem_init; a kernel
 * that waits for another workgroup must have all its workgroups resident.
 * Errors: NOT_INIT, INVALID_ARG. */
typedef struct {
    void *heap;          /* DEVICE: PE 0's segment                     */
    uint64_t seg;        /* bytes per PE segment                       */
    uint64_t *scratch;   /* DEVICE: the library's scratch words        */
    int npes;
} shmem_device_ctx;
typedef struct {
    uint64_t signals_off, counters_off;   /* byte offsets inside every segment */
    uint32_t nsignals, ncounters;
} shmem_gin_state;
int shmem_device_context(shmem_device_ctx *ctx_out /* HOST */);
int shmem_gin_device_state(void *gin, shmem_gin_state *state_out /* HOST */);

/* The unidirectional ring exchange of Listing 2, `rounds` times in one
 * persistent launch of npes * wgs_per_pe workgroups.  In each round PE r puts
 * bytes [peer*slot_bytes, +slot_bytes) of its send buffer (peer = (r+1) mod
 * npes) into bytes [r*slot_bytes, +slot_bytes) of the peer's receive buffer with
 * the actions SignalInc{signal_id} -- an atomic increment of the peer's signal
 * that lands only after the put is visible -- and CounterInc{counter_id}; then it
 * waits until its own signal reads 1 and its counter reads the round number,
 * resets the signal, and all PEs meet in the barrier session.  Afterwards every
 * signal and counter involved reads 0 again.  send_sym / recv_sym: symmetric,
 * npes * slot_bytes each, not overlapping.  The waits are bounded; a time-out
 * sets the device fault word.
 * Errors: NOT_INIT, INVALID_ARG (also: bad IDs, more workgroups than can be
 * co-resident), OUT_OF_RANGE, DEVICE. */
int shmem_ring_exchange(void *recv_sym, const void *send_sym, size_t slot_bytes, void *gin, int signal_id,
                        int counter_id, int rounds, int wgs_per_pe);

/* Put-with-signal ping-pong (the latency experiment of Sec. V-A) between PE 0
 * and PE 1, one workgroup each: PE 0 puts nbytes from its copy of buf_sym into
 * PE 1's copy with SignalInc{signal_id}; PE 1 waits, puts what it received into
 * PE 0's second buffer (buf_sym + nbytes rounded up to 256) with the same
 * action; `iters` round trips.  Signal `signal_id` must read 0 on PE 0 and PE 1
 * before the call and reads `iters` on both after it.  buf_sym spans
 * 2 * roundup(nbytes, 256) bytes.  Errors as above. */
int shmem_pingpong(void *buf_sym, size_t nbytes, void *gin, int signal_id, int iters);

/* Barrier epochs: in round e = 1..rounds every PE puts the value e into word
 * `pe` of slots_sym (uint64[npes], symmetric) on EVERY PE, all PEs meet in the
 * in-kernel barrier_all (quiet + synchronisation), and every PE checks that each
 * word of its own copy is at least e.  *dev_errors (DEVICE uint64, may be NULL)
 * is incremented once per violation; afterwards every word equals `rounds`.
 * Errors as above. */
int shmem_barrier_epochs(uint64_t *slots_sym, int rounds, int wgs_per_pe, uint64_t *dev_errors);

/* Teams of PEs: the members start, start + stride, ..., `size` of them (the
 * barrier session of Listing 1 takes a team; OpenSHMEM calls this an active
 * set).  shmem_team_create takes 256 bytes from the symmetric heap for the
 * team's arrival and generation words.  shmem_team_sync is the team's barrier
 * as one launch: quiet on the members, no member leaves before all have
 * arrived; PEs outside the team take no part (in stream order every earlier
 * call has completed anyway: the in-kernel form, pe_team_sync in
 * include/mi_shmem_device.hpp with the state from shmem_team_device_state, is
 * the one that matters).  shmem_team_epochs runs up to 8 DISJOINT teams side
 * by side in one persistent launch, team k for rounds[k] rounds: in round e
 * every member puts the value e into word (its index in the team) of
 * slots_sym (uint64[npes], symmetric) on every member, the team meets in its
 * barrier, and every member checks that each word of its own copy is at least
 * e; *dev_errors (DEVICE uint64, may be NULL) counts violations.  Afterwards
 * word i < size on every member of team k reads rounds[k]; PEs in no team are
 * untouched.
 * Errors: NOT_INIT, INVALID_ARG (also: overlapping teams, more workgroups than
 * can be co-resident), INVALID_PE (a member beyond npes), NOMEM, ALIGN,
 * OUT_OF_RANGE, DEVICE. */
typedef struct shmem_team *shmem_team_t;
typedef struct {
    uint32_t start, stride, size, pad;
    uint64_t words_off;          /* byte offset of the team's words in every segment */
} shmem_pe_team;
int shmem_team_create(int start, int stride, int size, shmem_team_t *team_out /* HOST */);
int shmem_team_destroy(shmem_team_t team);
int shmem_team_device_state(shmem_team_t team, shmem_pe_team *state_out /* HOST */);
int shmem_team_sync(shmem_team_t team, int wgs_per_pe);
int shmem_team_epochs(const shmem_team_t *teams /* HOST */, const int *rounds /* HOST */, int nteams,
                      uint64_t *slots_sym, int wgs_per_pe, uint64_t *dev_errors);

/* Message-passing litmus for fence and quiet (Sec. III-A "Ordering semantics":
 * what is put before the ordering point is visible to whoever sees what is put
 * after it).  PE 0 and PE 1, one workgroup each.  Round r = 1..rounds: PE 0
 * puts a block of nbytes (a multiple of 8) filled with r into PE 1's copy of
 * buf_sym, every wave calls fence (use_quiet = 0) or quiet (use_quiet = 1),
 * then one lane puts the flag word r and calls quiet; PE 1 polls the flag,
 * acquires, checks every word of the block and acknowledges.  *dev_errors
 * (DEVICE uint64, may be NULL) is incremented per word that was not r.
 * buf_sym spans roundup(nbytes, 256) + 512 bytes; the flag (at roundup(nbytes,
 * 256)) and the acknowledgement word (256 bytes further) must be 0 on both PEs
 * before the call and hold `rounds` after it.
 * Errors: NOT_INIT, INVALID_ARG (fewer than 2 PEs, rounds < 0, nbytes % 8),
 * ALIGN, OUT_OF_RANGE, DEVICE; a wait that times out surfaces at
 * shmem_stream_sync(). */
int shmem_fence_litmus(void *buf_sym, size_t nbytes, int rounds, int use_quiet, uint64_t *dev_errors);

/* -------------------------------------------------------------------------
 * MoE-shaped all-to-all in traffic shape: the low-latency dispatch / combine
 * of Sec. IV-E ("Low-Latency Kernel Integration") with the message sizes of
 * Sec. V-C (dispatch: 16 bytes of source-index metadata + the token; combine:
 * the token alone).  Payloads are opaque bytes; no quantisation, compression
 * or weighted floating-point reduction.
 *
 * num_experts experts are spread evenly over the PEs (expert e lives on PE
 * e / (num_experts / npes)).  Every PE holds up to max_tokens tokens of
 * hidden_bytes bytes, each routed to up to topk distinct experts.
 *
 * shmem_moe_create allocates, in the symmetric heap, the dispatch receive slots
 * ((num_experts/npes) * npes * max_tokens messages per PE), the combine slots
 * (max_tokens * topk tokens per PE) and 2 * num_experts + 8 64-bit words of
 * signals per PE (one per (local expert, sender) pair for the counts, one per
 * expert for the combine flags, eight for the library's own bookkeeping), and
 * clears the signals.  Limits: num_experts a multiple of npes and <= 1024,
 * max_tokens <= 128, topk <= 64, npes <= 256, hidden_bytes a positive
 * multiple of 16.  *moe_out is owned by the library until shmem_moe_destroy.
 * Errors: NOT_INIT, INVALID_ARG, NOMEM (heap too small), DEVICE. */
typedef struct shmem_moe *shmem_moe_t;
int shmem_moe_create(int num_experts, int max_tokens, int topk, size_t hidden_bytes, shmem_moe_t *moe_out);
int shmem_moe_destroy(shmem_moe_t moe);

/* One dispatch, asynchronous on the library's stream.  All arrays are DEVICE
 * memory owned by the caller, 16-byte aligned, with the PE as leading index:
 *   dev_x        const uint8 [npes][max_tokens][hidden_bytes]   tokens
 *   dev_topk     const int32 [npes][max_tokens][topk]  expert ids, < 0 = unused entry
 *   dev_ntok     const int32 [npes]                    tokens held by each PE
 *   dev_recv_x   uint8 [npes][E/npes][npes*max_tokens][hidden_bytes]  tokens received per local expert
 *   dev_recv_info int32 [npes][E/npes][npes*max_tokens][4]  per received token: source token
 *                index, source PE, position in the token's top-k list, expert id
 *   dev_recv_range int32 [npes][E/npes][npes][2]  (begin, count) of each sender's rows
 *   dev_recv_count int32 [npes][E/npes]           rows in use per local expert
 * Each sender writes one (metadata + token) message per route directly into a
 * slot at the expert's owner and then delivers the count of the (sender,
 * expert) pair with a zero-byte put + SignalAdd (release, then remote atomic
 * add of count + 1); receivers poll the signals, reset them and pack the
 * messages: senders in ascending PE order, a sender's tokens in ascending
 * order.  Rows beyond dev_recv_count are not written.  An expert id >=
 * num_experts or repeated within a token sets the device fault word
 * (shmem_stream_sync: BAD_TARGET / BAD_OP); that entry is skipped.  The waits
 * are bounded.  wgs_per_pe workgroups (of 512 threads) per PE must all be
 * co-resident: on an MI355X two fit a compute unit, i.e. npes * wgs_per_pe <=
 * 512 (INVALID_ARG beyond); one per compute unit measures best for batches of
 * 32 tokens per PE and more, one per local expert below.
 * Errors: NOT_INIT, INVALID_ARG, ALIGN, DEVICE. */
int shmem_moe_dispatch(shmem_moe_t moe, const void *dev_x, const int32_t *dev_topk, const int32_t *dev_ntok,
                       void *dev_recv_x, int32_t *dev_recv_info, int32_t *dev_recv_range, int32_t *dev_recv_count,
                       int wgs_per_pe);

/* One combine, asynchronous on the library's stream: row i of local expert le
 * on PE r in dev_expert_out (uint8, shaped like dev_recv_x) is sent to slot
 * (token, position) of the source PE named by dev_recv_info; after an expert's
 * rows one flag signal per destination follows the data (zero-byte put +
 * SignalAdd); each PE waits for the flags of a token's experts and writes
 *   dev_combined uint8 [npes][max_tokens][hidden_bytes]
 * = per token the sum, modulo 2^32 per 32-bit word, of the rows returned for
 * its valid routes (tokens at or beyond dev_ntok are not written).
 * dev_recv_info / dev_recv_range are the outputs of the matching dispatch;
 * dev_topk / dev_ntok are its inputs.  Flags count calls and are never reset.
 * Errors: as shmem_moe_dispatch. */
int shmem_moe_combine(shmem_moe_t moe, const void *dev_expert_out, const int32_t *dev_recv_info,
                      const int32_t *dev_recv_range, const int32_t *dev_topk, const int32_t *dev_ntok,
                      void *dev_combined, int wgs_per_pe);

/* -------------------------------------------------------------------------
 * Proxy-style executor (Sec. III-C, "Proxy Backend"): GPU threads enqueue the
 * 64-byte descriptors into a lock-free ring in pinned host memory with
 * fire-and-forget stores; one host thread per proxy object polls the ring,
 * validates each descriptor and carries it out on a stream of its own
 * (contiguous ops through the copy engine, strided ops with the library's
 * strided kernel), and publishes in GPU-visible memory how far it has got.
 * It is the second backend of the same descriptor format and a debugging twin
 * of shmem_op_batch: same table, same heap contents afterwards.
 *
 * shmem_proxy_create: queue_entries is a power of two in [2, 2^20] (a ring may
 * be much shorter than one submission, or than a wavefront); starts the thread.  shmem_proxy_submit: asynchronous; launches `workgroups` workgroups
 * (all must be co-resident) on the library's stream that enqueue dev_ops[0..n)
 * (DEVICE table, 16-byte aligned); descriptor i takes ticket (descriptors
 * submitted before) + i, so the ring order is the table order; producers wait
 * (bounded) while the ring is full.  The proxy carries descriptors out in
 * ticket order on one stream, i.e. in order -- stronger than the unordered
 * default of shmem_op_batch.  Work issued on the library's stream before the
 * submit happens before the proxy's copies of that submission; nothing orders
 * later work on the library's stream behind them except shmem_proxy_quiet.
 * shmem_proxy_quiet: blocks the calling host thread until every submitted
 * descriptor has been carried out and its copy is complete; returns
 * DEVICE_FAULT (and the ticket in *first_bad_index, may be NULL) if the proxy
 * rejected a descriptor (bad kind / PE / range / stride / alignment: skipped),
 * DEVICE if a producer timed out or a HIP call failed.
 * shmem_proxy_stats: counters so far (any pointer may be NULL).
 * shmem_proxy_destroy: waits for the library's stream, stops the thread, frees
 * the ring; shmem_finalize does the same for every proxy still alive.  One
 * caller thread per proxy object.
 * Errors: NOT_INIT, INVALID_ARG, ALIGN, NOMEM, DEVICE, DEVICE_FAULT. */
typedef struct shmem_proxy *shmem_proxy_t;
int shmem_proxy_create(size_t queue_entries, shmem_proxy_t *proxy_out);
int shmem_proxy_submit(shmem_proxy_t proxy, const void *dev_ops, size_t n, int workgroups);
int shmem_proxy_quiet(shmem_proxy_t proxy, uint64_t *first_bad_index);
int shmem_proxy_stats(shmem_proxy_t proxy, uint64_t *submitted, uint64_t *executed, uint64_t *rejected);
int shmem_proxy_destroy(shmem_proxy_t proxy);

/* Distributed transpose by one-sided gets (an iget-shaped variant; not in the
 * paper).  PE p holds rows [p*R, (p+1)*R), R = n / npes, of an n x n matrix of
 * elem_bytes-byte elements (4 or 8), row-major at in_sym; the call writes the
 * same rows of the transposed matrix at out_sym: B_p[i][j] = A_(j / R)[j % R][p*R + i].
 * The result is what npes * R * npes igets (source stride n, unit destination
 * stride) would produce; the kernel fetches 64 x 64 tiles with contiguous gets
 * and transposes them in LDS.  in_sym / out_sym: symmetric, R * n * elem_bytes
 * bytes each, not overlapping.  n must be a multiple of npes.  Asynchronous on
 * the library's stream; complete after shmem_quiet(-1) / shmem_barrier_all /
 * shmem_stream_sync.
 * Errors: NOT_INIT, INVALID_ARG, ALIGN, OUT_OF_RANGE, DEVICE. */
int shmem_transpose(void *out_sym, const void *in_sym, size_t n, size_t elem_bytes, int wgs_per_pe);

#ifdef __cplusplus
}
#endif
#endif

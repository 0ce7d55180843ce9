/*
 * CPU oracle for the one-sided (PGAS / OpenSHMEM-style) hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, single-threaded model of
 * what the path computes.  Processing elements are host arrays.  It shares no
 * code with the GPU library and must never be called from the product path;
 * only tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * Addressing: every buffer lives in the symmetric heap; an address is a byte
 * offset into a PE's segment ("window + offset", Sec. III-A "Windows-based
 * symmetric memory").  A "local" offset refers to the initiator's segment, a
 * "sym" offset to the segment of the PE the op names.
 *
 * Where the paper is silent (strided put, fetch-add / compare-swap return
 * values, fence, hash table, BFS) the ordinary OpenSHMEM meaning of the name
 * is taken; each function says which.
 */
#ifndef SHMEM_ORACLE_H
#define SHMEM_ORACLE_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct orc_world orc_world;

enum {
    ORC_OK = 0, ORC_ERR_INVALID_ARG = -3, ORC_ERR_INVALID_PE = -4,
    ORC_ERR_OUT_OF_RANGE = -5, ORC_ERR_ALIGN = -6, ORC_ERR_NOMEM = -7,
    ORC_ERR_BAD_FREE = -8
};

/* delivery modes for puts */
enum {
    ORC_DELIVER_EAGER = 0,    /* applied when issued                         */
    ORC_DELIVER_AT_QUIET = 1, /* buffered, applied at quiet in issue order   */
    ORC_DELIVER_SHUFFLED = 2  /* buffered, applied at quiet in a seeded
                                 random order that respects fences           */
};

orc_world *orc_init(int npes, size_t heap_bytes, int delivery_mode, uint64_t shuffle_seed);
void orc_finalize(orc_world *w);
int orc_n_pes(const orc_world *w);
size_t orc_heap_bytes(const orc_world *w);
uint8_t *orc_heap(orc_world *w, int pe);       /* host pointer to PE pe's segment */
size_t orc_pending(const orc_world *w, int pe);/* buffered deliveries of initiator pe */

/* symmetric allocator: same offset on every PE; -1 on failure / size 0 */
int64_t orc_malloc(orc_world *w, size_t nbytes);
int64_t orc_align(orc_world *w, size_t alignment, size_t nbytes);
int orc_free(orc_world *w, int64_t off);
size_t orc_live_blocks(const orc_world *w);

/* data movement */
int orc_put(orc_world *w, int pe_self, uint64_t dst_sym, uint64_t src_local, size_t nbytes, int pe);
int orc_put_value(orc_world *w, int pe_self, uint64_t dst_sym, uint64_t value, size_t nbytes, int pe);
int orc_get(orc_world *w, int pe_self, uint64_t dst_local, uint64_t src_sym, size_t nbytes, int pe);
int orc_iput(orc_world *w, int pe_self, uint64_t dst_sym, uint64_t src_local,
             int64_t dst_stride, int64_t src_stride, size_t nelems, size_t elem_bytes, int pe);
int orc_iget(orc_world *w, int pe_self, uint64_t dst_local, uint64_t src_sym,
             int64_t dst_stride, int64_t src_stride, size_t nelems, size_t elem_bytes, int pe);

/* 64-bit atomic memory operations; *old receives the previous value */
int orc_atomic_fetch_add(orc_world *w, int pe_self, uint64_t sym, uint64_t value, int pe, uint64_t *old);
int orc_atomic_compare_swap(orc_world *w, int pe_self, uint64_t sym, uint64_t cond, uint64_t value, int pe, uint64_t *old);
int orc_atomic_fetch_or(orc_world *w, int pe_self, uint64_t sym, uint64_t value, int pe, uint64_t *old);

/* ordering */
int orc_signal_add(orc_world *w, int pe_self, uint64_t sig_sym, uint64_t value, int pe);
int orc_fence(orc_world *w, int pe_self);
int orc_quiet(orc_world *w, int pe_self);
int orc_barrier_all(orc_world *w);
/* barrier over the PEs start, start + stride, ... (size members): quiet on the members only */
int orc_team_sync(orc_world *w, int start, int stride, int size);

/* 64-byte operation descriptor, same field layout as the generator's table */
typedef struct {
    uint32_t kind, pe_self, pe, elem_bytes;
    uint64_t local_off, sym_off, count;
    int64_t local_stride, sym_stride;
    uint64_t value;
} orc_op_desc;
enum { ORC_OP_PUT = 0, ORC_OP_GET = 1, ORC_OP_IPUT = 2, ORC_OP_IGET = 3 };

/* table executor: ops in index order, barrier_all after every quiet_every ops
 * and at the end; returns the first failing op's status or ORC_OK */
int orc_op_batch(orc_world *w, const orc_op_desc *ops, size_t n, size_t quiet_every);

/* batched AMOs on a symmetric counter array (uint64[T] per PE) */
enum { ORC_AMO_FETCH_ADD = 0, ORC_AMO_COMPARE_SWAP = 1, ORC_AMO_FETCH_OR = 2, ORC_AMO_MIN_CAS_LOOP = 3 };
int orc_amo_batch(orc_world *w, int kind, uint64_t ctr_sym, const int32_t *pe, const uint32_t *idx,
                  const uint64_t *a, const uint64_t *b, uint64_t *old, size_t n);

/* distributed open-addressing hash table (uint64 slots, 0 = empty) */
enum { ORC_HASH_INSERTED = 0, ORC_HASH_DUPLICATE = 1, ORC_HASH_FULL = 2 };
uint64_t orc_hash_mix64(uint64_t key);
int orc_hash_insert(orc_world *w, uint64_t table_sym, size_t slots_per_pe,
                    const uint64_t *keys, size_t n, uint8_t *status);
int orc_hash_lookup(orc_world *w, uint64_t table_sym, size_t slots_per_pe,
                    const uint64_t *keys, size_t n, uint8_t *found);

/* level-synchronous BFS over a 1D block vertex partition */
typedef struct {
    uint32_t nlevels;          /* number of non-empty frontiers (root's counts) */
    uint64_t reached;          /* vertices with level >= 0                      */
    uint64_t edges_traversed;  /* (sum of degrees of reached vertices) / 2      */
    uint64_t frontier_size[64];/* vertices per level, the first 64 levels       */
} orc_bfs_stats;
#define ORC_BFS_NONE 0xFFFFFFFFu
int orc_bfs(orc_world *w, uint32_t nverts, const uint64_t *row_off, const uint32_t *nbr,
            uint32_t root, int32_t *level, uint32_t *parent, orc_bfs_stats *stats);

#ifdef __cplusplus
}
#endif
#endif

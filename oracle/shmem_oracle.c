/*
 * CPU oracle for the one-sided hot path -- TEST INFRASTRUCTURE ONLY.
 * See shmem_oracle.h.  Plain C, single-threaded, no blocking, no fusion:
 * each function is the definition of its operation written out.
 */
#include "shmem_oracle.h"

#include <stdlib.h>
#include <string.h>

#define ORC_GRAN 256u /* allocator granularity and minimum alignment, bytes */

typedef struct { uint64_t off, len; } orc_block;

/* One buffered remote write.  A contiguous put is one element of nbytes. */
typedef struct {
    int pe;              /* target PE                                   */
    uint32_t epoch;      /* fence epoch of the initiator when issued    */
    uint64_t dst;        /* byte offset in the target's segment         */
    size_t elem_bytes, nelems;
    int64_t dst_stride;  /* in elements                                 */
    uint8_t *data;       /* packed snapshot of the source, or NULL ...  */
    uint64_t inl;        /* ... when the payload (<= 8 B) is held here  */
} orc_delivery;

typedef struct {
    orc_delivery *v; size_t n, cap; uint32_t epoch;
} orc_pendq;

struct orc_world {
    int npes; size_t heap_bytes; int mode; uint64_t rng;
    uint8_t **heap;
    orc_pendq *pend;
    orc_block *free_list; size_t nfree, capfree;   /* address-ordered */
    orc_block *live; size_t nlive, caplive;
};

/* ------------------------------------------------------------------ */
static uint64_t orc_rand(orc_world *w)
{   /* xorshift64*: only decides the order buffered puts are applied in */
    uint64_t x = w->rng;
    x ^= x >> 12; x ^= x << 25; x ^= x >> 27;
    w->rng = x;
    return x * 0x2545F4914F6CDD1Dull;
}

orc_world *orc_init(int npes, size_t heap_bytes, int delivery_mode, uint64_t shuffle_seed)
{
    if (npes < 1 || heap_bytes == 0 || heap_bytes % ORC_GRAN) return NULL;
    if (delivery_mode < ORC_DELIVER_EAGER || delivery_mode > ORC_DELIVER_SHUFFLED) return NULL;
    orc_world *w = (orc_world *)calloc(1, sizeof(*w));
    if (!w) return NULL;
    w->npes = npes; w->heap_bytes = heap_bytes; w->mode = delivery_mode;
    w->rng = shuffle_seed * 0x9E3779B97F4A7C15ull + 0x1234567ull;
    if (!w->rng) w->rng = 1;
    w->heap = (uint8_t **)calloc((size_t)npes, sizeof(uint8_t *));
    w->pend = (orc_pendq *)calloc((size_t)npes, sizeof(orc_pendq));
    for (int p = 0; p < npes; ++p) w->heap[p] = (uint8_t *)calloc(heap_bytes, 1);
    w->capfree = 16; w->free_list = (orc_block *)malloc(sizeof(orc_block) * w->capfree);
    w->free_list[0].off = 0; w->free_list[0].len = heap_bytes; w->nfree = 1;
    w->caplive = 16; w->live = (orc_block *)malloc(sizeof(orc_block) * w->caplive);
    return w;
}

static void orc_drop_pending(orc_pendq *q)
{
    for (size_t i = 0; i < q->n; ++i) free(q->v[i].data);
    q->n = 0;
}

void orc_finalize(orc_world *w)
{
    if (!w) return;
    for (int p = 0; p < w->npes; ++p) {
        orc_drop_pending(&w->pend[p]); free(w->pend[p].v); free(w->heap[p]);
    }
    free(w->heap); free(w->pend); free(w->free_list); free(w->live); free(w);
}

int orc_n_pes(const orc_world *w) { return w->npes; }
size_t orc_heap_bytes(const orc_world *w) { return w->heap_bytes; }
uint8_t *orc_heap(orc_world *w, int pe) { return (pe >= 0 && pe < w->npes) ? w->heap[pe] : NULL; }
size_t orc_pending(const orc_world *w, int pe) { return w->pend[pe].n; }
size_t orc_live_blocks(const orc_world *w) { return w->nlive; }

/* ------------------------------------------------------------------ */
/* Symmetric allocator.  One free list describes every PE's segment, so an
 * allocation has the same offset everywhere (same layout on all ranks,
 * Sec. III-A).  Policy (paper silent): address-ordered first fit, 256-byte
 * granularity, neighbours coalesced on free. */
static void orc_free_insert(orc_world *w, uint64_t off, uint64_t len)
{
    size_t i = 0;
    while (i < w->nfree && w->free_list[i].off < off) ++i;
    if (w->nfree == w->capfree) {
        w->capfree *= 2;
        w->free_list = (orc_block *)realloc(w->free_list, sizeof(orc_block) * w->capfree);
    }
    memmove(&w->free_list[i + 1], &w->free_list[i], sizeof(orc_block) * (w->nfree - i));
    w->free_list[i].off = off; w->free_list[i].len = len; w->nfree++;
    if (i + 1 < w->nfree && w->free_list[i].off + w->free_list[i].len == w->free_list[i + 1].off) {
        w->free_list[i].len += w->free_list[i + 1].len;
        memmove(&w->free_list[i + 1], &w->free_list[i + 2], sizeof(orc_block) * (w->nfree - i - 2));
        w->nfree--;
    }
    if (i > 0 && w->free_list[i - 1].off + w->free_list[i - 1].len == w->free_list[i].off) {
        w->free_list[i - 1].len += w->free_list[i].len;
        memmove(&w->free_list[i], &w->free_list[i + 1], sizeof(orc_block) * (w->nfree - i - 1));
        w->nfree--;
    }
}

int64_t orc_align(orc_world *w, size_t alignment, size_t nbytes)
{
    if (nbytes == 0 || alignment == 0 || (alignment & (alignment - 1))) return -1;
    if (alignment < ORC_GRAN) alignment = ORC_GRAN;
    uint64_t need = ((uint64_t)nbytes + ORC_GRAN - 1) / ORC_GRAN * ORC_GRAN;
    for (size_t i = 0; i < w->nfree; ++i) {
        uint64_t b = w->free_list[i].off, e = b + w->free_list[i].len;
        uint64_t a = (b + alignment - 1) / alignment * alignment;
        if (a + need > e || a + need < a) continue;
        /* take [a, a+need) out of free block i */
        memmove(&w->free_list[i], &w->free_list[i + 1], sizeof(orc_block) * (w->nfree - i - 1));
        w->nfree--;
        if (a > b) orc_free_insert(w, b, a - b);
        if (a + need < e) orc_free_insert(w, a + need, e - (a + need));
        if (w->nlive == w->caplive) {
            w->caplive *= 2;
            w->live = (orc_block *)realloc(w->live, sizeof(orc_block) * w->caplive);
        }
        w->live[w->nlive].off = a; w->live[w->nlive].len = need; w->nlive++;
        return (int64_t)a;
    }
    return -1;
}

int64_t orc_malloc(orc_world *w, size_t nbytes) { return orc_align(w, ORC_GRAN, nbytes); }

int orc_free(orc_world *w, int64_t off)
{
    if (off < 0) return ORC_ERR_BAD_FREE;
    for (size_t i = 0; i < w->nlive; ++i) {
        if (w->live[i].off == (uint64_t)off) {
            uint64_t len = w->live[i].len;
            w->live[i] = w->live[w->nlive - 1]; w->nlive--;
            orc_free_insert(w, (uint64_t)off, len);
            return ORC_OK;
        }
    }
    return ORC_ERR_BAD_FREE;
}

/* ------------------------------------------------------------------ */
static int orc_check_pe(const orc_world *w, int pe) { return pe >= 0 && pe < w->npes; }

static int orc_check_range(const orc_world *w, uint64_t off, uint64_t n)
{
    return off <= w->heap_bytes && n <= w->heap_bytes - off;
}

/* bytes spanned by nelems elements of eb bytes at a pitch of stride elements */
static int orc_check_strided(const orc_world *w, uint64_t off, int64_t stride, size_t nelems, size_t eb)
{
    if (nelems == 0) return off <= w->heap_bytes;
    if (stride < 1) return 0;
    uint64_t last = (uint64_t)(nelems - 1) * (uint64_t)stride;
    if (last / (uint64_t)stride != (uint64_t)(nelems - 1)) return 0;
    if (last > (UINT64_MAX - eb) / eb) return 0;
    return orc_check_range(w, off, last * eb + eb);
}

static void orc_apply(orc_world *w, const orc_delivery *d)
{
    const uint8_t *src = d->data ? d->data : (const uint8_t *)&d->inl;
    uint8_t *base = w->heap[d->pe] + d->dst;
    for (size_t i = 0; i < d->nelems; ++i)
        memcpy(base + (uint64_t)i * (uint64_t)d->dst_stride * d->elem_bytes,
               src + i * d->elem_bytes, d->elem_bytes);
}

/* Queue (or, in eager mode, apply) one remote write issued by pe_self. */
static void orc_post(orc_world *w, int pe_self, orc_delivery d)
{
    if (w->mode == ORC_DELIVER_EAGER) { orc_apply(w, &d); free(d.data); return; }
    orc_pendq *q = &w->pend[pe_self];
    if (q->n == q->cap) {
        q->cap = q->cap ? q->cap * 2 : 64;
        q->v = (orc_delivery *)realloc(q->v, sizeof(orc_delivery) * q->cap);
    }
    d.epoch = q->epoch;
    q->v[q->n++] = d;
}

/*
 * put: one-sided remote write, asynchronous (Sec. III-A "One-sided
 * communication semantics"; Table II put_nbi).  The source is read now -- it
 * is reusable on return -- and the bytes reach the target no later than the
 * initiator's next quiet / barrier.
 */
int orc_put(orc_world *w, int pe_self, uint64_t dst_sym, uint64_t src_local, size_t nbytes, int pe)
{
    if (!orc_check_pe(w, pe_self) || !orc_check_pe(w, pe)) return ORC_ERR_INVALID_PE;
    if (!orc_check_range(w, dst_sym, nbytes) || !orc_check_range(w, src_local, nbytes))
        return ORC_ERR_OUT_OF_RANGE;
    if (nbytes == 0) return ORC_OK; /* zero-byte put is legal and moves nothing (Sec. IV-C) */
    orc_delivery d; memset(&d, 0, sizeof d);
    d.pe = pe; d.dst = dst_sym; d.elem_bytes = nbytes; d.nelems = 1; d.dst_stride = 1;
    if (nbytes <= 8) memcpy(&d.inl, w->heap[pe_self] + src_local, nbytes);
    else { d.data = (uint8_t *)malloc(nbytes); memcpy(d.data, w->heap[pe_self] + src_local, nbytes); }
    orc_post(w, pe_self, d);
    return ORC_OK;
}

/* putValue: put of a small inline value, no source buffer (Listing 1). */
int orc_put_value(orc_world *w, int pe_self, uint64_t dst_sym, uint64_t value, size_t nbytes, int pe)
{
    if (!orc_check_pe(w, pe_self) || !orc_check_pe(w, pe)) return ORC_ERR_INVALID_PE;
    if (nbytes != 1 && nbytes != 2 && nbytes != 4 && nbytes != 8) return ORC_ERR_INVALID_ARG;
    if (!orc_check_range(w, dst_sym, nbytes)) return ORC_ERR_OUT_OF_RANGE;
    orc_delivery d; memset(&d, 0, sizeof d);
    d.pe = pe; d.dst = dst_sym; d.elem_bytes = nbytes; d.nelems = 1; d.dst_stride = 1;
    d.inl = value; /* little-endian host: the low nbytes are the payload */
    orc_post(w, pe_self, d);
    return ORC_OK;
}

/* get: blocking one-sided remote read (ordinary SHMEM meaning; paper names
 * get among the one-sided primitives, Sec. II). */
int orc_get(orc_world *w, int pe_self, uint64_t dst_local, uint64_t src_sym, size_t nbytes, int pe)
{
    if (!orc_check_pe(w, pe_self) || !orc_check_pe(w, pe)) return ORC_ERR_INVALID_PE;
    if (!orc_check_range(w, dst_local, nbytes) || !orc_check_range(w, src_sym, nbytes))
        return ORC_ERR_OUT_OF_RANGE;
    memmove(w->heap[pe_self] + dst_local, w->heap[pe] + src_sym, nbytes);
    return ORC_OK;
}

/* iput: dest[i*dst_stride] = src[i*src_stride], i < nelems, strides counted
 * in elements; bytes between elements are untouched (paper silent; ordinary
 * SHMEM meaning). */
int orc_iput(orc_world *w, int pe_self, uint64_t dst_sym, uint64_t src_local,
             int64_t dst_stride, int64_t src_stride, size_t nelems, size_t elem_bytes, int pe)
{
    if (!orc_check_pe(w, pe_self) || !orc_check_pe(w, pe)) return ORC_ERR_INVALID_PE;
    if (elem_bytes != 1 && elem_bytes != 2 && elem_bytes != 4 && elem_bytes != 8) return ORC_ERR_INVALID_ARG;
    if (dst_stride < 1 || src_stride < 1) return ORC_ERR_INVALID_ARG;
    if (dst_sym % elem_bytes || src_local % elem_bytes) return ORC_ERR_ALIGN;
    if (!orc_check_strided(w, dst_sym, dst_stride, nelems, elem_bytes) ||
        !orc_check_strided(w, src_local, src_stride, nelems, elem_bytes)) return ORC_ERR_OUT_OF_RANGE;
    if (nelems == 0) return ORC_OK;
    orc_delivery d; memset(&d, 0, sizeof d);
    d.pe = pe; d.dst = dst_sym; d.elem_bytes = elem_bytes; d.nelems = nelems; d.dst_stride = dst_stride;
    d.data = (uint8_t *)malloc(nelems * elem_bytes);
    for (size_t i = 0; i < nelems; ++i)
        memcpy(d.data + i * elem_bytes,
               w->heap[pe_self] + src_local + (uint64_t)i * (uint64_t)src_stride * elem_bytes, elem_bytes);
    orc_post(w, pe_self, d);
    return ORC_OK;
}

/* iget: the mirror of iput, blocking. */
int orc_iget(orc_world *w, int pe_self, uint64_t dst_local, uint64_t src_sym,
             int64_t dst_stride, int64_t src_stride, size_t nelems, size_t elem_bytes, int pe)
{
    if (!orc_check_pe(w, pe_self) || !orc_check_pe(w, pe)) return ORC_ERR_INVALID_PE;
    if (elem_bytes != 1 && elem_bytes != 2 && elem_bytes != 4 && elem_bytes != 8) return ORC_ERR_INVALID_ARG;
    if (dst_stride < 1 || src_stride < 1) return ORC_ERR_INVALID_ARG;
    if (dst_local % elem_bytes || src_sym % elem_bytes) return ORC_ERR_ALIGN;
    if (!orc_check_strided(w, dst_local, dst_stride, nelems, elem_bytes) ||
        !orc_check_strided(w, src_sym, src_stride, nelems, elem_bytes)) return ORC_ERR_OUT_OF_RANGE;
    for (size_t i = 0; i < nelems; ++i)
        memmove(w->heap[pe_self] + dst_local + (uint64_t)i * (uint64_t)dst_stride * elem_bytes,
                w->heap[pe] + src_sym + (uint64_t)i * (uint64_t)src_stride * elem_bytes, elem_bytes);
    return ORC_OK;
}

/* ------------------------------------------------------------------ */
/* Atomic memory operations on a remote 64-bit word (Table II "memory
 * atomics").  Applied at once and indivisibly in the oracle's serial
 * schedule; each returns the previous value (ordinary meaning). */
static int orc_amo_check(const orc_world *w, int pe_self, uint64_t sym, int pe)
{
    if (!orc_check_pe(w, pe_self) || !orc_check_pe(w, pe)) return ORC_ERR_INVALID_PE;
    if (sym % 8) return ORC_ERR_ALIGN;
    if (!orc_check_range(w, sym, 8)) return ORC_ERR_OUT_OF_RANGE;
    return ORC_OK;
}

int orc_atomic_fetch_add(orc_world *w, int pe_self, uint64_t sym, uint64_t value, int pe, uint64_t *old)
{
    int rc = orc_amo_check(w, pe_self, sym, pe); if (rc) return rc;
    uint64_t cur; memcpy(&cur, w->heap[pe] + sym, 8);
    uint64_t nxt = cur + value;                 /* wraps mod 2^64 */
    memcpy(w->heap[pe] + sym, &nxt, 8);
    if (old) *old = cur;
    return ORC_OK;
}

int orc_atomic_compare_swap(orc_world *w, int pe_self, uint64_t sym, uint64_t cond, uint64_t value, int pe, uint64_t *old)
{
    int rc = orc_amo_check(w, pe_self, sym, pe); if (rc) return rc;
    uint64_t cur; memcpy(&cur, w->heap[pe] + sym, 8);
    if (cur == cond) memcpy(w->heap[pe] + sym, &value, 8);
    if (old) *old = cur;
    return ORC_OK;
}

int orc_atomic_fetch_or(orc_world *w, int pe_self, uint64_t sym, uint64_t value, int pe, uint64_t *old)
{
    int rc = orc_amo_check(w, pe_self, sym, pe); if (rc) return rc;
    uint64_t cur; memcpy(&cur, w->heap[pe] + sym, 8);
    uint64_t nxt = cur | value;
    memcpy(w->heap[pe] + sym, &nxt, 8);
    if (old) *old = cur;
    return ORC_OK;
}

/* ------------------------------------------------------------------ */
/* fence: puts issued before it are delivered to a given PE before puts
 * issued after it to that same PE (ordinary SHMEM meaning; the paper's own
 * ordering rule is the per-peer put -> signal rule of Sec. III-A). */
int orc_fence(orc_world *w, int pe_self)
{
    if (!orc_check_pe(w, pe_self)) return ORC_ERR_INVALID_PE;
    w->pend[pe_self].epoch++;
    return ORC_OK;
}

/* Apply the buffered puts of initiator p that target PE `target` (-1: every
 * target), one fence epoch after the other, and drop them from the queue. */
static void orc_deliver(orc_world *w, int p, int target)
{
    orc_pendq *q = &w->pend[p];
    size_t i = 0;
    while (i < q->n) {                       /* one run per fence epoch */
        size_t j = i;
        while (j < q->n && q->v[j].epoch == q->v[i].epoch) ++j;
        if (w->mode == ORC_DELIVER_SHUFFLED)
            for (size_t k = j - 1; k > i; --k) {
                size_t r = i + (size_t)(orc_rand(w) % (uint64_t)(k - i + 1));
                orc_delivery t = q->v[k]; q->v[k] = q->v[r]; q->v[r] = t;
            }
        for (size_t k = i; k < j; ++k)
            if (target < 0 || q->v[k].pe == target) orc_apply(w, &q->v[k]);
        i = j;
    }
    size_t keep = 0;
    for (size_t k = 0; k < q->n; ++k) {
        if (target < 0 || q->v[k].pe == target) free(q->v[k].data);
        else q->v[keep++] = q->v[k];
    }
    q->n = keep;
    if (keep == 0) q->epoch = 0;
}

static void orc_quiet_one(orc_world *w, int p) { orc_deliver(w, p, -1); }

/* signal: remote atomic add on a 64-bit signal word.  When it completes at
 * the destination, every earlier put of this initiator to that peer is
 * visible there (Sec. III-A "Ordering semantics"); puts to other peers stay
 * buffered. */
int orc_signal_add(orc_world *w, int pe_self, uint64_t sig_sym, uint64_t value, int pe)
{
    int rc = orc_amo_check(w, pe_self, sig_sym, pe); if (rc) return rc;
    orc_deliver(w, pe_self, pe);
    return orc_atomic_fetch_add(w, pe_self, sig_sym, value, pe, NULL);
}

/* quiet: every earlier put of the caller is complete and visible to all PEs
 * (Table II quiet; the stronger, SHMEM reading -- unlike flush, which only
 * promises the source is reusable, Sec. III-A "Ordering semantics").
 * pe_self = -1 means every PE. */
int orc_quiet(orc_world *w, int pe_self)
{
    if (pe_self == -1) { for (int p = 0; p < w->npes; ++p) orc_quiet_one(w, p); return ORC_OK; }
    if (!orc_check_pe(w, pe_self)) return ORC_ERR_INVALID_PE;
    orc_quiet_one(w, pe_self);
    return ORC_OK;
}

/* barrier_all: quiet on every PE, then all PEs are synchronised (Table II
 * barrier; Sec. III-B "Barrier synchronization"). */
int orc_barrier_all(orc_world *w) { return orc_quiet(w, -1); }

/* Barrier over a team of PEs -- the members start, start + stride, ... (size of them), the way the
 * paper's barrier session takes a team (Listing 1; Sec. III-B "Barrier synchronization") and
 * OpenSHMEM names an active set: quiet on every MEMBER, then the members are synchronised.  What
 * the other PEs have issued stays where it is. */
int orc_team_sync(orc_world *w, int start, int stride, int size)
{
    if (start < 0 || stride < 1 || size < 1) return ORC_ERR_INVALID_ARG;
    if ((long long)start + (long long)(size - 1) * stride >= w->npes) return ORC_ERR_INVALID_PE;
    for (int i = 0; i < size; ++i) orc_quiet_one(w, start + i * stride);
    return ORC_OK;
}

/* ------------------------------------------------------------------ */
int orc_op_batch(orc_world *w, const orc_op_desc *ops, size_t n, size_t quiet_every)
{
    int first = ORC_OK;
    for (size_t i = 0; i < n; ++i) {
        const orc_op_desc *d = &ops[i];
        int rc;
        switch (d->kind) {
        case ORC_OP_PUT: rc = orc_put(w, (int)d->pe_self, d->sym_off, d->local_off, d->count, (int)d->pe); break;
        case ORC_OP_GET: rc = orc_get(w, (int)d->pe_self, d->local_off, d->sym_off, d->count, (int)d->pe); break;
        case ORC_OP_IPUT: rc = orc_iput(w, (int)d->pe_self, d->sym_off, d->local_off, d->sym_stride,
                                        d->local_stride, d->count, d->elem_bytes, (int)d->pe); break;
        case ORC_OP_IGET: rc = orc_iget(w, (int)d->pe_self, d->local_off, d->sym_off, d->local_stride,
                                        d->sym_stride, d->count, d->elem_bytes, (int)d->pe); break;
        default: rc = ORC_ERR_INVALID_ARG;
        }
        if (rc && !first) first = rc;
        if (quiet_every && (i + 1) % quiet_every == 0) orc_barrier_all(w);
    }
    orc_barrier_all(w);
    return first;
}

/* ------------------------------------------------------------------ */
/* Op i is issued by PE i / ceil(n / npes) (block layout).  The issuer does
 * not influence any result. */
static int orc_issuer(const orc_world *w, size_t i, size_t n)
{
    size_t per = (n + (size_t)w->npes - 1) / (size_t)w->npes;
    return (int)(i / per);
}

int orc_amo_batch(orc_world *w, int kind, uint64_t ctr_sym, const int32_t *pe, const uint32_t *idx,
                  const uint64_t *a, const uint64_t *b, uint64_t *old, size_t n)
{
    for (size_t i = 0; i < n; ++i) {
        int me = orc_issuer(w, i, n);
        uint64_t addr = ctr_sym + 8ull * idx[i], seen = 0;
        int rc;
        switch (kind) {
        case ORC_AMO_FETCH_ADD: rc = orc_atomic_fetch_add(w, me, addr, a[i], pe[i], &seen); break;
        case ORC_AMO_COMPARE_SWAP: rc = orc_atomic_compare_swap(w, me, addr, a[i], b[i], pe[i], &seen); break;
        case ORC_AMO_FETCH_OR: rc = orc_atomic_fetch_or(w, me, addr, a[i], pe[i], &seen); break;
        case ORC_AMO_MIN_CAS_LOOP: {
            /* store a[i] if the word is 0 or larger, by a compare-swap retry loop */
            uint64_t cur;
            rc = orc_atomic_fetch_add(w, me, addr, 0, pe[i], &cur);   /* atomic fetch */
            while (!rc && (cur == 0 || cur > a[i])) {
                rc = orc_atomic_compare_swap(w, me, addr, cur, a[i], pe[i], &seen);
                if (seen == cur) break;
                cur = seen;
            }
            seen = cur;
            break;
        }
        default: rc = ORC_ERR_INVALID_ARG;
        }
        if (rc) return rc;
        if (old) old[i] = seen;
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------ */
/* 64-bit avalanche mixer used as the hash function (paper silent; this is
 * the finaliser of the public-domain SplitMix64 generator). */
uint64_t orc_hash_mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* insert: owner = h mod npes; home = (h / npes) mod slots; linear probing
 * inside the owner's table; each probe is compare_swap(slot, 0, key). */
int orc_hash_insert(orc_world *w, uint64_t table_sym, size_t slots_per_pe,
                    const uint64_t *keys, size_t n, uint8_t *status)
{
    if (slots_per_pe == 0) return ORC_ERR_INVALID_ARG;
    for (size_t i = 0; i < n; ++i) {
        uint64_t key = keys[i];
        if (key == 0) return ORC_ERR_INVALID_ARG;
        uint64_t h = orc_hash_mix64(key);
        int owner = (int)(h % (uint64_t)w->npes);
        uint64_t home = (h / (uint64_t)w->npes) % slots_per_pe;
        int me = orc_issuer(w, i, n);
        uint8_t st = ORC_HASH_FULL;
        for (uint64_t j = 0; j < slots_per_pe; ++j) {
            uint64_t slot = (home + j) % slots_per_pe, seen;
            int rc = orc_atomic_compare_swap(w, me, table_sym + 8 * slot, 0, key, owner, &seen);
            if (rc) return rc;
            if (seen == 0) { st = ORC_HASH_INSERTED; break; }
            if (seen == key) { st = ORC_HASH_DUPLICATE; break; }
        }
        if (status) status[i] = st;
    }
    return ORC_OK;
}

/* lookup: same probe sequence with 8-byte gets until the key or an empty slot. */
int orc_hash_lookup(orc_world *w, uint64_t table_sym, size_t slots_per_pe,
                    const uint64_t *keys, size_t n, uint8_t *found)
{
    if (slots_per_pe == 0) return ORC_ERR_INVALID_ARG;
    int64_t land = orc_malloc(w, 8);           /* landing word for the gets */
    if (land < 0) return ORC_ERR_NOMEM;
    int rc = ORC_OK;
    for (size_t i = 0; i < n && !rc; ++i) {
        uint64_t key = keys[i];
        uint64_t h = orc_hash_mix64(key);
        int owner = (int)(h % (uint64_t)w->npes);
        uint64_t home = (h / (uint64_t)w->npes) % slots_per_pe;
        int me = orc_issuer(w, i, n);
        uint8_t f = 0;
        for (uint64_t j = 0; j < slots_per_pe; ++j) {
            uint64_t slot = (home + j) % slots_per_pe, seen;
            rc = orc_get(w, me, (uint64_t)land, table_sym + 8 * slot, 8, owner);
            if (rc) break;
            memcpy(&seen, w->heap[me] + land, 8);
            if (seen == key) { f = 1; break; }
            if (seen == 0) break;
        }
        found[i] = f;
    }
    orc_free(w, land);
    return rc;
}

/* ------------------------------------------------------------------ */
/*
 * Level-synchronous BFS, 1D block partition: owner(v) = v / vpp with
 * vpp = ceil(nverts / npes).  Per PE, in the symmetric heap: a visited bitmap
 * (uint64 words), level (int32), parent (uint32), two frontier queues
 * (uint32) and their two tails (uint64).  A vertex is claimed by fetch_or on
 * its owner's bitmap; the claimer reserves a queue slot with fetch_add on the
 * owner's next tail and puts v, parent and level there.
 */
int orc_bfs(orc_world *w, uint32_t nverts, const uint64_t *row_off, const uint32_t *nbr,
            uint32_t root, int32_t *level, uint32_t *parent, orc_bfs_stats *stats)
{
    if (nverts == 0 || root >= nverts) return ORC_ERR_INVALID_ARG;
    const int npes = w->npes;
    const uint32_t vpp = (uint32_t)(((uint64_t)nverts + (uint64_t)npes - 1) / (uint64_t)npes);
    const uint64_t words = ((uint64_t)vpp + 63) / 64;
    int64_t bm = orc_malloc(w, words * 8), lv = orc_malloc(w, (size_t)vpp * 4),
            pr = orc_malloc(w, (size_t)vpp * 4), q0 = orc_malloc(w, (size_t)vpp * 4),
            q1 = orc_malloc(w, (size_t)vpp * 4), tl = orc_malloc(w, 16);
    int rc = ORC_OK;
    if (bm < 0 || lv < 0 || pr < 0 || q0 < 0 || q1 < 0 || tl < 0) { rc = ORC_ERR_NOMEM; goto done; }
    const uint64_t q[2] = { (uint64_t)q0, (uint64_t)q1 };
    memset(stats, 0, sizeof *stats);

    for (int p = 0; p < npes; ++p) {           /* each owner initialises its slice */
        memset(w->heap[p] + bm, 0, words * 8);
        memset(w->heap[p] + lv, 0xFF, (size_t)vpp * 4);   /* level  = -1   */
        memset(w->heap[p] + pr, 0xFF, (size_t)vpp * 4);   /* parent = NONE */
        memset(w->heap[p] + tl, 0, 16);
    }
    {   /* the root's owner seeds the search */
        int o = (int)(root / vpp); uint32_t l = root % vpp;
        uint64_t bit = 1ull << (l % 64), one = 1; int32_t zero = 0;
        uint64_t word; memcpy(&word, w->heap[o] + bm + 8 * (l / 64), 8); word |= bit;
        memcpy(w->heap[o] + bm + 8 * (l / 64), &word, 8);
        memcpy(w->heap[o] + lv + 4 * (uint64_t)l, &zero, 4);
        memcpy(w->heap[o] + pr + 4 * (uint64_t)l, &root, 4);
        memcpy(w->heap[o] + q[0], &root, 4);
        memcpy(w->heap[o] + tl, &one, 8);
    }

    int cur = 0; uint32_t L = 0;
    for (;;) {
        uint64_t total = 0;
        for (int p = 0; p < npes; ++p) { uint64_t t; memcpy(&t, w->heap[p] + tl + 8 * cur, 8); total += t; }
        if (total == 0) break;
        if (L < 64) stats->frontier_size[L] = total;   /* the record holds the first 64 levels; nlevels counts all */
        for (int p = 0; p < npes; ++p) {
            uint64_t cnt; memcpy(&cnt, w->heap[p] + tl + 8 * cur, 8);
            for (uint64_t k = 0; k < cnt; ++k) {
                uint32_t u; memcpy(&u, w->heap[p] + q[cur] + 4 * k, 4);
                for (uint64_t e = row_off[u]; e < row_off[u + 1]; ++e) {
                    uint32_t v = nbr[e];
                    int o = (int)(v / vpp); uint32_t l = v % vpp;
                    uint64_t bit = 1ull << (l % 64), seen, slot;
                    orc_atomic_fetch_or(w, p, (uint64_t)bm + 8 * (l / 64), bit, o, &seen);
                    if (seen & bit) continue;
                    orc_atomic_fetch_add(w, p, (uint64_t)tl + 8 * (1 - cur), 1, o, &slot);
                    orc_put_value(w, p, q[1 - cur] + 4 * slot, v, 4, o);
                    orc_put_value(w, p, (uint64_t)pr + 4 * (uint64_t)l, u, 4, o);
                    orc_put_value(w, p, (uint64_t)lv + 4 * (uint64_t)l, (uint64_t)(L + 1), 4, o);
                }
            }
        }
        orc_barrier_all(w);
        for (int p = 0; p < npes; ++p) memset(w->heap[p] + tl + 8 * cur, 0, 8);
        cur = 1 - cur; ++L;
    }
    stats->nlevels = L;
    for (uint32_t v = 0; v < nverts; ++v) {
        int o = (int)(v / vpp); uint32_t l = v % vpp;
        memcpy(&level[v], w->heap[o] + lv + 4 * (uint64_t)l, 4);
        memcpy(&parent[v], w->heap[o] + pr + 4 * (uint64_t)l, 4);
        if (level[v] >= 0) { stats->reached++; stats->edges_traversed += row_off[v + 1] - row_off[v]; }
    }
    stats->edges_traversed /= 2;
done:
    if (bm >= 0) orc_free(w, bm);
    if (lv >= 0) orc_free(w, lv);
    if (pr >= 0) orc_free(w, pr);
    if (q0 >= 0) orc_free(w, q0);
    if (q1 >= 0) orc_free(w, q1);
    if (tl >= 0) orc_free(w, tl);
    return rc;
}

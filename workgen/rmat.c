/*
 * Seeded R-MAT edge generator and CSR builder (input generation only).
 *
 * This file produces INPUT ARRAYS for the BFS workload; it holds none of the
 * BFS method's arithmetic.  Both the CPU oracle and the GPU path consume the
 * arrays it writes.
 *
 * Recipe (stands in for the scale-24 / edge-factor-16 / (0.57,0.19,0.19)
 * problem class; it is not that benchmark's generator):
 *   - edge e, bit level l: one 64-bit draw from a counter-based generator
 *     keyed by (seed, e, l) picks a quadrant with probabilities (a,b,c,d)
 *     and sets bit l of (src,dst) accordingly; no per-level noise;
 *   - vertices are relabelled through a seeded Fisher-Yates permutation;
 *   - self-loops are dropped, duplicate edges are kept;
 *   - every kept edge is stored in both directions;
 *   - CSR neighbour order = order of a stable counting sort by source over
 *     the sequence (e0 fwd, e0 rev, e1 fwd, e1 rev, ...).
 * Edges are i.i.d. by construction, so no separate edge shuffle is applied.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <pthread.h>

/* Counter-based generator: a 64-bit avalanche mixer over (seed, counter). */
static inline uint64_t wg_draw(uint64_t seed, uint64_t ctr)
{
    uint64_t x = seed ^ (ctr * 0xD6E8FEB86659FD93ull);
    x ^= x >> 33; x *= 0xFF51AFD7ED558CCDull;
    x ^= x >> 33; x *= 0xC4CEB9FE1A85EC53ull;
    x ^= x >> 33;
    return x;
}

typedef struct {
    int scale; uint64_t nedges; uint64_t seed;
    uint64_t ta, tb, tc;           /* cumulative thresholds on a 2^53 grid */
    const uint32_t *perm;
    uint32_t *src, *dst;
    uint64_t e0, e1;
} gen_job;

static void *gen_worker(void *p)
{
    gen_job *j = (gen_job *)p;
    for (uint64_t e = j->e0; e < j->e1; ++e) {
        uint32_t s = 0, d = 0;
        for (int l = 0; l < j->scale; ++l) {
            uint64_t u = wg_draw(j->seed, e * 64u + (uint64_t)l) >> 11; /* 53 bits */
            if (u < j->ta) { /* quadrant a: neither bit */ }
            else if (u < j->tb) d |= 1u << l;        /* b: column bit  */
            else if (u < j->tc) s |= 1u << l;        /* c: row bit     */
            else { s |= 1u << l; d |= 1u << l; }     /* d: both bits   */
        }
        j->src[e] = j->perm[s];
        j->dst[e] = j->perm[d];
    }
    return NULL;
}

/* Writes nedges (src,dst) pairs, relabelled unless relabel == 0 (the raw
 * labels exist so that tests can check the per-bit quadrant frequencies). */
int wg_rmat_edges(int scale, uint64_t nedges, double a, double b, double c,
                  uint64_t seed, int nthreads, int relabel, uint32_t *src, uint32_t *dst)
{
    if (scale < 1 || scale > 31 || nthreads < 1) return -1;
    uint64_t n = 1ull << scale;
    uint32_t *perm = (uint32_t *)malloc(n * sizeof(uint32_t));
    if (!perm) return -2;
    for (uint64_t i = 0; i < n; ++i) perm[i] = (uint32_t)i;
    for (uint64_t i = n - 1; relabel && i > 0; --i) {  /* Fisher-Yates */
        uint64_t r = wg_draw(seed ^ 0xA5A5A5A55A5A5A5Aull, i) % (i + 1);
        uint32_t t = perm[i]; perm[i] = perm[r]; perm[r] = t;
    }
    const double grid = 9007199254740992.0;          /* 2^53 */
    pthread_t *th = (pthread_t *)malloc(sizeof(pthread_t) * nthreads);
    gen_job *jobs = (gen_job *)malloc(sizeof(gen_job) * nthreads);
    for (int t = 0; t < nthreads; ++t) {
        gen_job *j = &jobs[t];
        j->scale = scale; j->nedges = nedges; j->seed = seed;
        j->ta = (uint64_t)(a * grid);
        j->tb = (uint64_t)((a + b) * grid);
        j->tc = (uint64_t)((a + b + c) * grid);
        j->perm = perm; j->src = src; j->dst = dst;
        j->e0 = nedges * (uint64_t)t / nthreads;
        j->e1 = nedges * (uint64_t)(t + 1) / nthreads;
        pthread_create(&th[t], NULL, gen_worker, j);
    }
    for (int t = 0; t < nthreads; ++t) pthread_join(th[t], NULL);
    free(jobs); free(th); free(perm);
    return 0;
}

typedef struct {
    uint64_t nedges; const uint32_t *src, *dst;
    uint32_t v0, v1;                 /* this worker owns sources in [v0, v1) */
    uint64_t *cursor;                /* per-vertex write cursor (starts at row offset) */
    uint32_t *nbr;
} fill_job;

static void *fill_worker(void *p)
{
    fill_job *j = (fill_job *)p;
    for (uint64_t e = 0; e < j->nedges; ++e) {
        uint32_t s = j->src[e], d = j->dst[e];
        if (s == d) continue;
        if (s >= j->v0 && s < j->v1) j->nbr[j->cursor[s]++] = d;
        if (d >= j->v0 && d < j->v1) j->nbr[j->cursor[d]++] = s;
    }
    return NULL;
}

/*
 * Pass 1 (nbr == NULL): fills row_off[0..n] and returns the number of CSR
 * entries through *nnz.  Pass 2 (nbr != NULL): fills nbr[0..nnz).
 */
int wg_csr_build(uint32_t nverts, uint64_t nedges, const uint32_t *src,
                 const uint32_t *dst, int nthreads, uint64_t *row_off,
                 uint32_t *nbr, uint64_t *nnz)
{
    if (nthreads < 1) return -1;
    if (!nbr) {
        memset(row_off, 0, sizeof(uint64_t) * ((size_t)nverts + 1));
        for (uint64_t e = 0; e < nedges; ++e) {
            uint32_t s = src[e], d = dst[e];
            if (s >= nverts || d >= nverts) return -3;
            if (s == d) continue;
            row_off[(size_t)s + 1]++; row_off[(size_t)d + 1]++;
        }
        for (uint32_t v = 0; v < nverts; ++v) row_off[(size_t)v + 1] += row_off[v];
        *nnz = row_off[nverts];
        return 0;
    }
    uint64_t *cursor = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)nverts);
    if (!cursor) return -2;
    memcpy(cursor, row_off, sizeof(uint64_t) * (size_t)nverts);
    pthread_t *th = (pthread_t *)malloc(sizeof(pthread_t) * nthreads);
    fill_job *jobs = (fill_job *)malloc(sizeof(fill_job) * nthreads);
    for (int t = 0; t < nthreads; ++t) {
        fill_job *j = &jobs[t];
        j->nedges = nedges; j->src = src; j->dst = dst;
        j->v0 = (uint32_t)((uint64_t)nverts * t / nthreads);
        j->v1 = (uint32_t)((uint64_t)nverts * (t + 1) / nthreads);
        j->cursor = cursor; j->nbr = nbr;
        pthread_create(&th[t], NULL, fill_worker, j);
    }
    for (int t = 0; t < nthreads; ++t) pthread_join(th[t], NULL);
    free(jobs); free(th); free(cursor);
    return 0;
}

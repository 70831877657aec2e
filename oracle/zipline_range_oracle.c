/*
 * CPU oracle for the ZipLine search under the paper's formal objective
 * (ElasticBSP, arXiv 2001.01347, Section III "The Problem": d_Z = max(Z) -
 * min(Z), the waiting time of the fastest worker; Section IV, Algorithm 2).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, host-only C.  It shares no code,
 * header, table or helper with the HIP library; the product path never calls
 * it.
 *
 * What is computed.  One instance is a P x R matrix t[p][i] of predicted end
 * timestamps, every row non-decreasing.  A set Z holds one timestamp of every
 * worker; d_Z = max(Z) - min(Z).  For a barrier time c the tightest such set
 * takes every worker's latest timestamp at or before c:
 *
 *   last_p(c) = max{ t[p][i] : t[p][i] <= c }
 *   d(c)      = c - min_p last_p(c)              (c itself is some last_p(c))
 *   C         = { t[p][i] } with c >= max_p t[p][0]
 *   d*        = min_{c in C} d(c)
 *   barrier*  = the smallest c in C with d(c) = d*   (Fig. 3 caption: of
 *               several equal minima the first is taken; Algorithm 2 updates
 *               on strict "<" only)
 *   iters[p]  = #{ i : t[p][i] <= barrier* }
 *
 * Four routes, so that each can pin the others:
 *   zl_range_naive       Section IV "Naive search": all R^P choices Z, value
 *                        max(Z) - min(Z), ties to the smaller max(Z).
 *   zl_range_definition  the formulas above written out.
 *   zl_range_latest      the sweep of Algorithm 2 with a table of every worker's
 *                        latest timestamp: the merged timestamps are visited in
 *                        ascending order, equal values together; after the
 *                        group at value c the table holds last_p(c), and once
 *                        every worker has an entry d(c) = c - (smallest entry)
 *                        is a candidate.  The smallest entry is found by
 *                        looking through the table, O(n) per candidate as in
 *                        the paper's complexity count (Table I).
 *   zl_range_sweep       the same sweep with the oldest of the latest timestamps
 *                        kept at the head of a queue (timestamps enter the table in
 *                        ascending order, so its entries in order of arrival are sorted);
 *                        O(n log n) for the sort, used for large instances.
 *
 * Readings where the paper is silent: a barrier time is a candidate only once
 * every worker has a timestamp at or before it (Fig. 3 caption: the set must
 * hold all n workers); timestamps that are equal count together, in whatever
 * order they are stored (the value at such a time is the one with all of them
 * taken in).
 *
 * Return value of every routine: 0 on success, 1 if a row is not
 * non-decreasing (outputs untouched), 2 on invalid arguments.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int range_rows_sorted(const int64_t *t, int32_t P, int32_t R)
{
    for (int32_t p = 0; p < P; ++p)
        for (int32_t i = 1; i < R; ++i)
            if (t[(size_t)p * R + i] < t[(size_t)p * R + i - 1])
                return 0;
    return 1;
}

static void range_count_iters(const int64_t *t, int32_t P, int32_t R, int64_t barrier, int32_t *iters)
{
    for (int32_t p = 0; p < P; ++p) {
        int32_t c = 0;
        for (int32_t i = 0; i < R; ++i)
            if (t[(size_t)p * R + i] <= barrier)
                ++c;
        iters[p] = c;
    }
}

/* differences of int64 timestamps as unsigned 64-bit numbers (max - min >= 0) */
static uint64_t span_of(int64_t hi, int64_t lo) { return (uint64_t)hi - (uint64_t)lo; }

/* ------------------------------------------------------------------ */
/* Section IV "Naive search": every combination of one element per worker. */
int zl_range_naive(const int64_t *t, int32_t P, int32_t R,
                   int64_t *barrier, int32_t *iters, int64_t *dmin)
{
    if (!t || P < 1 || R < 1 || !barrier || !iters || !dmin)
        return 2;
    if (!range_rows_sorted(t, P, R))
        return 1;
    int32_t *idx = (int32_t *)calloc((size_t)P, sizeof(int32_t));
    if (!idx)
        return 2;
    int have = 0;
    uint64_t best_d = 0;
    int64_t best_max = 0;
    for (;;) {
        int64_t mx = t[idx[0]], mn = t[idx[0]];
        for (int32_t p = 1; p < P; ++p) {
            const int64_t v = t[(size_t)p * R + idx[p]];
            if (v > mx) mx = v;
            if (v < mn) mn = v;
        }
        const uint64_t d = span_of(mx, mn);
        if (!have || d < best_d || (d == best_d && mx < best_max)) {
            have = 1;
            best_d = d;
            best_max = mx;
        }
        int32_t p = 0;                      /* next combination (odometer) */
        while (p < P && ++idx[p] == R)
            idx[p++] = 0;
        if (p == P)
            break;
    }
    free(idx);
    *barrier = best_max;
    *dmin = (int64_t)best_d;
    range_count_iters(t, P, R, best_max, iters);
    return 0;
}

/* ------------------------------------------------------------------ */
/* The definition written out: every admissible candidate c, every worker's
 * latest timestamp at or before c. */
int zl_range_definition(const int64_t *t, int32_t P, int32_t R,
                        int64_t *barrier, int32_t *iters, int64_t *dmin)
{
    if (!t || P < 1 || R < 1 || !barrier || !iters || !dmin)
        return 2;
    if (!range_rows_sorted(t, P, R))
        return 1;
    int64_t first_all = t[0];               /* max_p t[p][0] */
    for (int32_t p = 1; p < P; ++p)
        if (t[(size_t)p * R] > first_all)
            first_all = t[(size_t)p * R];
    int have = 0;
    uint64_t best_d = 0;
    int64_t best_c = 0;
    for (int32_t q = 0; q < P; ++q)
        for (int32_t j = 0; j < R; ++j) {
            const int64_t c = t[(size_t)q * R + j];
            if (c < first_all)
                continue;
            int64_t lowest = c;
            for (int32_t p = 0; p < P; ++p) {
                int64_t last = t[(size_t)p * R];          /* exists: c >= every first */
                for (int32_t i = 1; i < R; ++i)
                    if (t[(size_t)p * R + i] <= c)
                        last = t[(size_t)p * R + i];
                if (last < lowest)
                    lowest = last;
            }
            const uint64_t d = span_of(c, lowest);
            if (!have || d < best_d || (d == best_d && c < best_c)) {
                have = 1;
                best_d = d;
                best_c = c;
            }
        }
    *barrier = best_c;
    *dmin = (int64_t)best_d;
    range_count_iters(t, P, R, best_c, iters);
    return 0;
}

/* ------------------------------------------------------------------ */
typedef struct { int64_t v; int32_t p; } relem_t;

static int relem_cmp(const void *a, const void *b)
{
    const relem_t *x = (const relem_t *)a, *y = (const relem_t *)b;
    if (x->v != y->v)
        return x->v < y->v ? -1 : 1;
    return (x->p > y->p) - (x->p < y->p);
}

static relem_t *merged_sorted(const int64_t *t, int32_t P, int32_t R)
{
    const size_t n = (size_t)P * R;
    relem_t *om = (relem_t *)malloc(n * sizeof(relem_t));
    if (!om)
        return NULL;
    for (int32_t p = 0; p < P; ++p)
        for (int32_t i = 0; i < R; ++i) {
            om[(size_t)p * R + i].v = t[(size_t)p * R + i];
            om[(size_t)p * R + i].p = p;
        }
    qsort(om, n, sizeof(relem_t), relem_cmp);
    return om;
}

/* The sweep with an explicit table of the workers' latest timestamps (Algorithm 2; of several equal
 * minima the first, Fig. 3 caption). */
int zl_range_latest(const int64_t *t, int32_t P, int32_t R,
                    int64_t *barrier, int32_t *iters, int64_t *dmin)
{
    if (!t || P < 1 || R < 1 || !barrier || !iters || !dmin)
        return 2;
    if (!range_rows_sorted(t, P, R))
        return 1;
    const size_t n = (size_t)P * R;
    relem_t *om = merged_sorted(t, P, R);
    int64_t *latest = (int64_t *)malloc((size_t)P * sizeof(int64_t));
    char *started = (char *)calloc((size_t)P, 1);
    if (!om || !latest || !started) {
        free(om); free(latest); free(started);
        return 2;
    }
    int32_t nstarted = 0;                   /* workers that have a timestamp <= c */
    int have = 0;
    uint64_t best_d = 0;
    int64_t best_c = 0;
    size_t i = 0;
    while (i < n) {
        const int64_t c = om[i].v;
        for (; i < n && om[i].v == c; ++i) {            /* every timestamp equal to c */
            const int32_t p = om[i].p;
            if (!started[p]) { started[p] = 1; ++nstarted; }
            latest[p] = c;
        }
        if (nstarted < P)
            continue;                                   /* c lies before some worker's first timestamp */
        int64_t oldest = latest[0];
        for (int32_t p = 1; p < P; ++p)
            if (latest[p] < oldest) oldest = latest[p];
        const uint64_t d = span_of(c, oldest);
        if (!have || d < best_d) {                      /* candidates come in ascending order: the first minimum stays */
            have = 1;
            best_d = d;
            best_c = c;
        }
    }
    free(om); free(latest); free(started);
    if (!have)
        return 2;
    *barrier = best_c;
    *dmin = (int64_t)best_d;
    range_count_iters(t, P, R, best_c, iters);
    return 0;
}

/* The same sweep for large instances.  Timestamps enter the table in ascending
 * order, so its entries in order of arrival are sorted and the oldest one is the
 * earliest arrival that has not been replaced: a queue of arrivals with a
 * "replaced" mark.  d is evaluated after every arrival once every worker has
 * an entry; at equal timestamps the later evaluations can only be smaller and
 * the strict comparison takes them, so the result is d at the last of them. */
int zl_range_sweep(const int64_t *t, int32_t P, int32_t R,
                   int64_t *barrier, int32_t *iters, int64_t *dmin)
{
    if (!t || P < 1 || R < 1 || !barrier || !iters || !dmin)
        return 2;
    if (!range_rows_sorted(t, P, R))
        return 1;
    const size_t n = (size_t)P * R;
    relem_t *om = merged_sorted(t, P, R);
    size_t *slot = (size_t *)malloc((size_t)P * sizeof(size_t));   /* queue position of worker p's entry */
    char *inZ = (char *)calloc((size_t)P, 1);
    char *replaced = (char *)calloc(n, 1);
    if (!om || !slot || !inZ || !replaced) {
        free(om); free(slot); free(inZ); free(replaced);
        return 2;
    }
    size_t head = 0;                        /* the queue is om[head..k] minus the replaced ones */
    int32_t size = 0;
    int have = 0;
    uint64_t best_d = 0;
    int64_t best_max = 0;
    for (size_t k = 0; k < n; ++k) {
        const int32_t p = om[k].p;
        if (inZ[p]) replaced[slot[p]] = 1; else { inZ[p] = 1; ++size; }
        slot[p] = k;
        if (size < P)
            continue;
        while (replaced[head])
            ++head;
        const uint64_t d = span_of(om[k].v, om[head].v);
        if (!have || d < best_d) {
            have = 1;
            best_d = d;
            best_max = om[k].v;
        }
    }
    free(om); free(slot); free(inZ); free(replaced);
    if (!have)
        return 2;
    *barrier = best_max;
    *dmin = (int64_t)best_d;
    range_count_iters(t, P, R, best_max, iters);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Batch driver: ts[B][P][R] -> barrier[B], iters[B][P], dmin[B].
 * method: 0 sweep, 1 definition, 2 naive, 3 zipline (Algorithm 2 as printed). */
int zl_range_batch(const int64_t *ts, int64_t B, int32_t P, int32_t R,
                   int64_t *barrier, int32_t *iters, int64_t *dmin,
                   int32_t *rc, int32_t method, int32_t threads,
                   int32_t *threads_used)
{
    if (!ts || B < 1 || P < 1 || R < 1 || !barrier || !iters || !dmin ||
        method < 0 || method > 3)
        return 2;
    int worst = 0;
    int used = 1;
#ifdef _OPENMP
    if (threads > 0)
        omp_set_num_threads(threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#pragma omp parallel for schedule(dynamic, 1) reduction(max : worst)
#endif
    for (int64_t b = 0; b < B; ++b) {
        const int64_t *t = ts + (size_t)b * P * R;
        int32_t *it = iters + (size_t)b * P;
        int r;
        if (method == 0)
            r = zl_range_sweep(t, P, R, barrier + b, it, dmin + b);
        else if (method == 1)
            r = zl_range_definition(t, P, R, barrier + b, it, dmin + b);
        else if (method == 2)
            r = zl_range_naive(t, P, R, barrier + b, it, dmin + b);
        else
            r = zl_range_latest(t, P, R, barrier + b, it, dmin + b);
        if (rc)
            rc[b] = r;
        if (r > worst)
            worst = r;
    }
    if (threads_used)
        *threads_used = used;
    return worst;
}

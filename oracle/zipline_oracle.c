/*
 * CPU oracle for the ZipLine barrier search (ElasticBSP, arXiv 2001.01347).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, host-only C.  It shares no code,
 * header, table or helper with the HIP library; the product path never calls
 * it.  Only the tests, the smoke check and the benchmark's CPU-baseline leg
 * may load this file's shared object.
 *
 * What is computed (Section III "The Problem", with the objective read as the
 * summed waiting time that Fig. 1's caption, Section I and the Conclusion
 * describe: the barrier at which the overall waiting time of all workers is
 * least).  One instance is a P x R matrix t[p][i] of predicted end
 * timestamps, every row non-decreasing in i (Section IV, matrix M):
 *
 *   last_p(c) = max{ t[p][i] : t[p][i] <= c }
 *   wait(c)   = sum_p ( c - last_p(c) )
 *   C         = { t[p][i] } with c >= max_p t[p][0]   (every worker has
 *               finished at least one iteration: Algorithm 2's initial fill
 *               of Z until all n workers are present)
 *   wait*     = min_{c in C} wait(c)
 *   barrier*  = the smallest c in C with wait(c) = wait*   (Fig. 3 caption:
 *               of several equal minima the first one is taken; Algorithm 2
 *               updates on strict "<" only)
 *   iters[p]  = #{ i : t[p][i] <= barrier* }
 *
 * Three independent routes to that result are kept so that each can pin the
 * others:
 *   zl_oracle_naive       Section IV "Naive search": every one of the R^P
 *                         choices Z of one timestamp per worker, value
 *                         sum_p (max Z - z_p); tiny inputs only.
 *   zl_oracle_definition  the formulas above written out, O((P R)^2 R).
 *   zl_oracle_sweep       Algorithm 2's order of work: sort the merged set
 *                         Omega, sweep it left to right keeping in Z the
 *                         newest timestamp of every worker, evaluate once all
 *                         workers are present, keep the first minimum.
 *
 * Readings where the paper is silent: timestamps equal across workers are
 * all admitted by a barrier at that time, so a candidate is evaluated only
 * after every element with the same value has entered Z; sums are carried in
 * 128-bit integers and the results are returned as int64 (the caller's
 * precondition is P * (max t - min t) <= INT64_MAX).
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

typedef __int128 wide_t;

static int rows_sorted(const int64_t *t, int32_t P, int32_t R)
{
    for (int32_t p = 0; p < P; ++p)
        for (int32_t i = 1; i < R; ++i)
            if (t[(size_t)p * R + i] < t[(size_t)p * R + i - 1])
                return 0;
    return 1;
}

/* iters[p] = number of entries of row p that are <= barrier (linear count). */
static void count_iters(const int64_t *t, int32_t P, int32_t R, int64_t barrier,
                        int32_t *iters)
{
    for (int32_t p = 0; p < P; ++p) {
        int32_t n = 0;
        for (int32_t i = 0; i < R; ++i)
            if (t[(size_t)p * R + i] <= barrier)
                ++n;
        iters[p] = n;
    }
}

/* ------------------------------------------------------------------ */
/* Section IV, "Naive search": all R^P choices, summed-wait objective. */
int zl_oracle_naive(const int64_t *t, int32_t P, int32_t R,
                    int64_t *barrier, int32_t *iters, int64_t *wait)
{
    if (!t || P < 1 || R < 1 || !barrier || !iters || !wait)
        return 2;
    if (!rows_sorted(t, P, R))
        return 1;
    int32_t *j = (int32_t *)calloc((size_t)P, sizeof(int32_t));
    if (!j)
        return 2;
    int have = 0;
    wide_t best_val = 0;
    int64_t best_bar = 0;
    for (;;) {
        /* Z = { t[p][j[p]] }: barrier is max Z, every worker waits max Z - z_p. */
        int64_t mx = t[(size_t)0 * R + j[0]];
        for (int32_t p = 1; p < P; ++p)
            if (t[(size_t)p * R + j[p]] > mx)
                mx = t[(size_t)p * R + j[p]];
        wide_t val = 0;
        for (int32_t p = 0; p < P; ++p)
            val += (wide_t)mx - (wide_t)t[(size_t)p * R + j[p]];
        if (!have || val < best_val || (val == best_val && mx < best_bar)) {
            have = 1;
            best_val = val;
            best_bar = mx;
        }
        /* next choice (odometer over the P indices) */
        int32_t p = 0;
        while (p < P) {
            if (++j[p] < R)
                break;
            j[p] = 0;
            ++p;
        }
        if (p == P)
            break;
    }
    free(j);
    *barrier = best_bar;
    *wait = (int64_t)best_val;
    count_iters(t, P, R, best_bar, iters);
    return 0;
}

/* ------------------------------------------------------------------ */
/* The definition written out: every timestamp is tried as the barrier. */
int zl_oracle_definition(const int64_t *t, int32_t P, int32_t R,
                         int64_t *barrier, int32_t *iters, int64_t *wait)
{
    if (!t || P < 1 || R < 1 || !barrier || !iters || !wait)
        return 2;
    if (!rows_sorted(t, P, R))
        return 1;
    int64_t thr = t[0];
    for (int32_t p = 1; p < P; ++p)
        if (t[(size_t)p * R] > thr)
            thr = t[(size_t)p * R];
    int have = 0;
    wide_t best_val = 0;
    int64_t best_bar = 0;
    for (size_t k = 0; k < (size_t)P * R; ++k) {
        int64_t c = t[k];
        if (c < thr)
            continue;
        wide_t w = 0;
        for (int32_t p = 0; p < P; ++p) {
            /* last_p(c): the largest entry of row p that is <= c; it exists
               because c >= thr >= t[p][0]. */
            int64_t last = t[(size_t)p * R];
            for (int32_t i = 0; i < R; ++i) {
                int64_t v = t[(size_t)p * R + i];
                if (v <= c && v > last)
                    last = v;
            }
            w += (wide_t)c - (wide_t)last;
        }
        if (!have || w < best_val || (w == best_val && c < best_bar)) {
            have = 1;
            best_val = w;
            best_bar = c;
        }
    }
    *barrier = best_bar;
    *wait = (int64_t)best_val;
    count_iters(t, P, R, best_bar, iters);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Algorithm 2's order of work: sort Omega, sweep, first minimum wins.  */
typedef struct {
    int64_t t;
    int32_t p;
} elem_t;

static int elem_cmp(const void *a, const void *b)
{
    const elem_t *x = (const elem_t *)a, *y = (const elem_t *)b;
    if (x->t < y->t)
        return -1;
    if (x->t > y->t)
        return 1;
    return (x->p > y->p) - (x->p < y->p);
}

int zl_oracle_sweep(const int64_t *t, int32_t P, int32_t R,
                    int64_t *barrier, int32_t *iters, int64_t *wait)
{
    if (!t || P < 1 || R < 1 || !barrier || !iters || !wait)
        return 2;
    if (!rows_sorted(t, P, R))
        return 1;
    size_t n = (size_t)P * R;
    elem_t *omega = (elem_t *)malloc(n * sizeof(elem_t));
    int64_t *z = (int64_t *)malloc((size_t)P * sizeof(int64_t));
    char *in_z = (char *)calloc((size_t)P, 1);
    if (!omega || !z || !in_z) {
        free(omega);
        free(z);
        free(in_z);
        return 2;
    }
    /* Omega: the merged set of all workers' timestamps, sorted ascending. */
    for (int32_t p = 0; p < P; ++p)
        for (int32_t i = 0; i < R; ++i) {
            omega[(size_t)p * R + i].t = t[(size_t)p * R + i];
            omega[(size_t)p * R + i].p = p;
        }
    qsort(omega, n, sizeof(elem_t), elem_cmp);

    int32_t present = 0; /* |Z| */
    wide_t sum_z = 0;    /* sum of the elements of Z */
    int have = 0;
    wide_t best_val = 0;
    int64_t best_bar = 0;
    size_t k = 0;
    while (k < n) {
        int64_t c = omega[k].t;
        /* take every element with this value: each replaces its worker's
           older element in Z (or enters Z if the worker was absent). */
        while (k < n && omega[k].t == c) {
            int32_t p = omega[k].p;
            if (in_z[p])
                sum_z -= (wide_t)z[p];
            else {
                in_z[p] = 1;
                ++present;
            }
            z[p] = c;
            sum_z += (wide_t)c;
            ++k;
        }
        if (present == P) {
            wide_t w = (wide_t)P * (wide_t)c - sum_z; /* sum_p (c - z_p) */
            if (!have || w < best_val) {              /* strict: first minimum */
                have = 1;
                best_val = w;
                best_bar = c;
            }
        }
    }
    free(omega);
    free(z);
    free(in_z);
    *barrier = best_bar;
    *wait = (int64_t)best_val;
    count_iters(t, P, R, best_bar, iters);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Batch driver: ts[B][P][R] -> barrier[B], iters[B][P], wait[B].
 * method: 0 sweep, 1 definition, 2 naive.  threads <= 0: library default.
 * rc[b] (may be NULL) receives each instance's return value; the function
 * returns the largest of them.  Returns the number of threads actually used
 * through *threads_used (may be NULL). */
int zl_oracle_batch(const int64_t *ts, int64_t B, int32_t P, int32_t R,
                    int64_t *barrier, int32_t *iters, int64_t *wait,
                    int32_t *rc, int32_t method, int32_t threads,
                    int32_t *threads_used)
{
    if (!ts || B < 1 || P < 1 || R < 1 || !barrier || !iters || !wait ||
        method < 0 || method > 2)
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
        int r;
        if (method == 0)
            r = zl_oracle_sweep(t, P, R, barrier + b, iters + (size_t)b * P, wait + b);
        else if (method == 1)
            r = zl_oracle_definition(t, P, R, barrier + b, iters + (size_t)b * P, wait + b);
        else
            r = zl_oracle_naive(t, P, R, barrier + b, iters + (size_t)b * P, wait + b);
        if (rc)
            rc[b] = r;
        if (r > worst)
            worst = r;
    }
    if (threads_used)
        *threads_used = used;
    return worst;
}

/* ------------------------------------------------------------------ */
/* The entry point declared in include/ebsp_zipline_oracle.h: the sweep
 * route over a batch, host pointers, `threads` worker threads (<= 0: the
 * library default).  Returns 0, or the largest per-instance code (1: some
 * row of some instance is not non-decreasing, its outputs stay untouched;
 * 2: invalid arguments). */
int ebsp_zipline_oracle(const int64_t *ts, int64_t B, int32_t P, int32_t R,
                        int64_t *barrier, int32_t *iters, int64_t *wait, int32_t threads)
{
    return zl_oracle_batch(ts, B, P, R, barrier, iters, wait, NULL, 0, threads, NULL);
}

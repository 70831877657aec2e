/*
 * CPU oracle for GridScan and FullGridScan (ElasticBSP, arXiv 2001.01347,
 * Section IV "GridScan", Algorithm 1, and the paragraph "FullGridScan").
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, host-only C; shares nothing with
 * the HIP library, and the product path never calls it.
 *
 * What is computed.  One instance is the n x R matrix M of predicted end
 * timestamps, every row non-decreasing (Section IV).  For a designated
 * point e (one entry of a designated row) the set Z holds e and, from each
 * other row, the point at the shortest distance |M[p][i] - e| to e;
 * d_Z = max(Z) - min(Z) (Section III).
 *   GridScan      designates the row whose first timestamp is the smallest,
 *                 forms Z for each of its R points in order, and keeps the
 *                 Z with the smallest d_Z (replaced on strict "<" only).
 *   FullGridScan  does the same with every row in turn as the designated
 *                 row and keeps the smallest d_Z over all n*R sets.
 * Returned: dz = d_Z*, barrier = max(Z*), iters[p] = 1 + the index in row p
 * of the point that Z* holds (what Algorithm 1 returns, as counts).
 *
 * Readings where the paper is silent: of two points of a row at the same
 * distance from e the earlier one is taken (the first found by a scan from
 * the left that replaces on strict "<"; this also picks the first of equal
 * timestamps); of several rows with the same smallest first timestamp the
 * first is designated; FullGridScan takes the rows in index order, so of
 * equal minima the one met first in (row, point) order is kept.
 *
 * Two routes: gs_scan follows the order of work of Algorithm 1 (every point
 * of every other row is looked at: O(R^2 n) and O(R^2 n^2)); gs_bisect finds
 * the nearest point by bisection in the sorted row and is used for inputs the
 * first route would take too long for; each pins the other on small inputs.
 *
 * Return value: 0 on success, 1 if a row is not non-decreasing (outputs
 * untouched), 2 on invalid arguments.
 */
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef __int128 wide_t;

static int gs_rows_sorted(const int64_t *t, int32_t P, int32_t R)
{
    for (int32_t p = 0; p < P; ++p)
        for (int32_t i = 1; i < R; ++i)
            if (t[(size_t)p * R + i] < t[(size_t)p * R + i - 1])
                return 0;
    return 1;
}

static wide_t gs_dist(int64_t a, int64_t b)
{
    wide_t d = (wide_t)a - (wide_t)b;
    return d < 0 ? -d : d;
}

/* Index of the point of `row` nearest to e: every point is looked at. */
static int32_t nearest_scan(const int64_t *row, int32_t R, int64_t e)
{
    int32_t best = 0;
    wide_t bd = gs_dist(row[0], e);
    for (int32_t i = 1; i < R; ++i) {
        wide_t d = gs_dist(row[i], e);
        if (d < bd) {
            bd = d;
            best = i;
        }
    }
    return best;
}

/* The same by bisection: the last point below e and the first point at or
 * above it are the only candidates; the earlier one wins a tie, and of equal
 * timestamps the first. */
static int32_t first_at_or_above(const int64_t *row, int32_t R, int64_t v)
{
    int32_t lo = 0, hi = R;
    while (lo < hi) {
        int32_t m = lo + (hi - lo) / 2;
        if (row[m] < v)
            lo = m + 1;
        else
            hi = m;
    }
    return lo;
}

static int32_t nearest_bisect(const int64_t *row, int32_t R, int64_t e)
{
    int32_t up = first_at_or_above(row, R, e);
    if (up == 0)
        return 0;
    int32_t down = first_at_or_above(row, R, row[up - 1]); /* first of the equal timestamps below e */
    if (up == R)
        return down;
    return gs_dist(row[down], e) <= gs_dist(row[up], e) ? down : up;
}

/* One designated row: Z for each of its points; *have / best_* carry the
 * smallest d_Z so far across calls. */
static void scan_designated(const int64_t *t, int32_t P, int32_t R, int32_t pb, int bisect,
                            int *have, wide_t *best_d, int32_t *best_row, int32_t *best_point)
{
    for (int32_t j = 0; j < R; ++j) {
        int64_t e = t[(size_t)pb * R + j];
        int64_t mx = e, mn = e;
        for (int32_t p = 0; p < P; ++p) {
            if (p == pb)
                continue;
            const int64_t *row = t + (size_t)p * R;
            int32_t i = bisect ? nearest_bisect(row, R, e) : nearest_scan(row, R, e);
            if (row[i] > mx)
                mx = row[i];
            if (row[i] < mn)
                mn = row[i];
        }
        wide_t d = (wide_t)mx - (wide_t)mn;
        if (!*have || d < *best_d) {
            *have = 1;
            *best_d = d;
            *best_row = pb;
            *best_point = j;
        }
    }
}

static int gs_search(const int64_t *t, int32_t P, int32_t R, int full, int bisect,
                     int64_t *barrier, int32_t *iters, int64_t *dz)
{
    if (!t || P < 1 || R < 1 || !barrier || !iters || !dz)
        return 2;
    if (!gs_rows_sorted(t, P, R))
        return 1;
    int have = 0;
    wide_t best_d = 0;
    int32_t best_row = 0, best_point = 0;
    if (full) {
        for (int32_t pb = 0; pb < P; ++pb)
            scan_designated(t, P, R, pb, bisect, &have, &best_d, &best_row, &best_point);
    } else {
        int32_t pb = 0; /* the row with the smallest first timestamp */
        for (int32_t p = 1; p < P; ++p)
            if (t[(size_t)p * R] < t[(size_t)pb * R])
                pb = p;
        scan_designated(t, P, R, pb, bisect, &have, &best_d, &best_row, &best_point);
    }
    /* Z* again, to return it */
    int64_t e = t[(size_t)best_row * R + best_point];
    int64_t mx = e;
    for (int32_t p = 0; p < P; ++p) {
        const int64_t *row = t + (size_t)p * R;
        int32_t i = p == best_row ? best_point
                                  : (bisect ? nearest_bisect(row, R, e) : nearest_scan(row, R, e));
        iters[p] = i + 1;
        if (row[i] > mx)
            mx = row[i];
    }
    *barrier = mx;
    *dz = (int64_t)best_d;
    return 0;
}

/* Batch driver: ts[B][P][R] -> barrier[B], iters[B][P], dz[B].  full: 0 GridScan,
 * 1 FullGridScan.  method: 0 every point looked at, 1 bisection.  rc[b] (may be
 * NULL) receives each instance's return value; returns the largest of them. */
int gs_batch(const int64_t *ts, int64_t B, int32_t P, int32_t R, int32_t full, int32_t method,
             int64_t *barrier, int32_t *iters, int64_t *dz, int32_t *rc, int32_t threads,
             int32_t *threads_used)
{
    if (!ts || B < 1 || P < 1 || R < 1 || !barrier || !iters || !dz || method < 0 || method > 1)
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
        int r = gs_search(ts + (size_t)b * P * R, P, R, full != 0, method, barrier + b,
                          iters + (size_t)b * P, dz + b);
        if (rc)
            rc[b] = r;
        if (r > worst)
            worst = r;
    }
    if (threads_used)
        *threads_used = used;
    return worst;
}

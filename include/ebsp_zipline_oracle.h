/*
 * ebsp_zipline_oracle.h -- C entry point of the CPU oracle of the ZipLine
 * barrier search.  TEST INFRASTRUCTURE: the oracle is a separate host-only
 * library (oracle/libzipline_oracle.so, plain C, no HIP), shares no code with
 * libebsp_zipline.so, and is loaded only by the tests, the smoke check and the
 * benchmark's CPU-baseline leg.
 *
 * What it computes (ElasticBSP, arXiv 2001.01347): Section III "The Problem"
 * with the objective read as the summed waiting time of all workers (Fig. 1's
 * caption, Section I, the Conclusion); of the routes the oracle keeps (Section
 * IV "Naive search" over all R^P choices, the definition written out, and the
 * order of work of Algorithm 2: sort the merged set, sweep it once keeping
 * every worker's newest timestamp, first minimum wins) this entry point runs
 * the last one.  Per instance, with last_p(c) = max{ t[p][i] <= c }:
 *
 *     wait    = min over timestamps c >= max_p t[p][0] of sum_p (c - last_p(c)),
 *     barrier = the smallest such c, iters[p] = #{ i : t[p][i] <= barrier }.
 *
 * All pointers are HOST pointers owned by the caller.
 *   ts       in   [B][P][R] int64 row-major, every row non-decreasing
 *   barrier  out  [B]; iters out [B][P] (1..R); wait out [B]
 *   threads       worker threads over the instances (<= 0: the library default)
 * Returns 0 on success, 1 if some instance has a row that is not
 * non-decreasing (that instance's outputs are left untouched, the others are
 * written), 2 on invalid arguments (NULL pointer, B, P or R < 1).
 */
#ifndef EBSP_ZIPLINE_ORACLE_H
#define EBSP_ZIPLINE_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

int ebsp_zipline_oracle(const int64_t* ts, int64_t B, int32_t P, int32_t R,
                        int64_t* barrier, int32_t* iters, int64_t* wait, int32_t threads);

#ifdef __cplusplus
}
#endif
#endif /* EBSP_ZIPLINE_ORACLE_H */

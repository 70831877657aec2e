/*
 * ebsp_zipline.h -- C ABI of the MI355X (gfx950) ZipLine barrier search.
 *
 * The operation (Section III "The Problem" and Algorithm 2 of the ElasticBSP
 * paper, arXiv 2001.01347, with the objective read as the summed waiting time
 * of all workers that Fig. 1's caption, Section I and the Conclusion describe):
 * one instance is a P x R matrix t[p][i] of predicted iteration end
 * timestamps, row p non-decreasing in i.  For a barrier time c let
 * last_p(c) = max{ t[p][i] <= c }.  Over all timestamps c with
 * c >= max_p t[p][0] (every worker has finished an iteration: Algorithm 2's
 * initial fill of Z) the search returns
 *
 *     wait    = min_c  sum_p ( c - last_p(c) ),
 *     barrier = the smallest c that attains it (Fig. 3 caption: the first of
 *               several equal minima),
 *     iters[p]= #{ i : t[p][i] <= barrier }   (the per-worker iteration counts
 *               of the superstep, Fig. 1 caption).
 *
 * All data pointers are DEVICE pointers owned by the caller.  The calls only
 * enqueue work on `stream` (a hipStream_t passed as void*); they never
 * synchronise it, never allocate and never free.  The caller keeps every
 * buffer alive until the stream has passed the call.  Calls on different
 * streams may overlap if they use different workspaces.  A call records
 * kernel launches only (no memory set or copy nodes), so a stream may be
 * captured into a HIP graph around it; the first call on a device also asks the
 * runtime for the device's name, so make one call before capturing.
 *
 * Tuning knobs, per-kernel timing and the bandwidth yardsticks that the
 * benchmark uses are declared in ebsp_zipline_bench.h.
 */
#ifndef EBSP_ZIPLINE_H
#define EBSP_ZIPLINE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Return codes.  Nothing is enqueued when an error is returned, except for
 * EBSP_ERR_LAUNCH, which may follow earlier launches of the same call. */
#define EBSP_OK                0
#define EBSP_ERR_NULL         -1   /* a required pointer is NULL                         */
#define EBSP_ERR_SHAPE        -2   /* B < 0, P < 1, R < 1, or P*R >= 2^31                */
#define EBSP_ERR_WORKSPACE    -3   /* workspace_bytes < ebsp_zipline_workspace_bytes()   */
#define EBSP_ERR_LAUNCH       -4   /* the HIP runtime refused a launch; see last_error   */
#define EBSP_ERR_DEVICE       -5   /* the current HIP device is not a gfx950             */

/* Per-instance status bits written to status[b] (data errors; that instance's
 * outputs are then unspecified, other instances are unaffected). */
#define EBSP_STATUS_OK         0
#define EBSP_STATUS_UNSORTED   1   /* some row is not non-decreasing (Section III: rows  */
                                   /* are iteration sequences)                            */
#define EBSP_STATUS_OVERFLOW   2   /* P * (max t - min t) does not fit in int64          */

/*
 * Bytes of device scratch that ebsp_zipline_batch needs for this shape.
 * Returns 0 for invalid shapes and for shapes that need no scratch (small
 * instances are handled by one workgroup each, entirely in LDS).
 * ebsp_predict_zipline_workspace_bytes is the same for
 * ebsp_predict_zipline_batch (predicted rows take other kernels, which need
 * more scratch).
 */
size_t ebsp_zipline_workspace_bytes(int64_t B, int32_t P, int32_t R);
size_t ebsp_predict_zipline_workspace_bytes(int64_t B, int32_t P, int32_t R);

/*
 * Batched ZipLine search: B independent instances.
 *
 *   ts        in   [B][P][R] int64, row-major, device; timestamps in any fixed
 *                  unit and epoch (microseconds in the paper's setting); every
 *                  row non-decreasing.  Not modified.
 *   barrier   out  [B] int64, device; same unit and epoch as ts.
 *   iters     out  [B][P] int32, device; 1..R.
 *   wait      out  [B] int64, device; >= 0.
 *   status    out  [B] int32, device, or NULL; EBSP_STATUS_* bits.
 *   workspace      device scratch of at least ebsp_zipline_workspace_bytes()
 *                  bytes, 256-byte aligned (may be NULL when that is 0).  Its
 *                  contents are undefined before and after the call.
 *   stream         hipStream_t (as void*); NULL is the default stream.
 *
 * Precondition per instance: P * (max t - min t) <= INT64_MAX.  B == 0 is a
 * valid no-op.  Outputs of valid instances are fully overwritten.
 * Returns EBSP_OK or a negative EBSP_ERR_* code.
 */
int ebsp_zipline_batch(const int64_t* ts, int64_t B, int32_t P, int32_t R,
                       int64_t* barrier, int32_t* iters, int64_t* wait,
                       int32_t* status, void* workspace, size_t workspace_bytes,
                       void* stream);

/*
 * ebsp_zipline_batch for callers that cannot allocate device memory or pass a
 * workspace (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): the same search, the same arguments without the
 * workspace, the same results.  The scratch is a device array of
 * EBSP_STATIC_SCRATCH_BYTES bytes inside the library, held by every GPU the
 * library runs on until the process ends; its address on the current device
 * is looked up on the first call there and kept.  The call allocates and frees
 * nothing and only enqueues kernels on `stream`.
 * A batch whose ebsp_zipline_workspace_bytes() exceeds the array is refused
 * with EBSP_ERR_WORKSPACE (nothing enqueued; ebsp_last_error() says how much
 * it needs): split it over several calls.  All calls on one GPU share the one
 * array, so calls that overlap on a GPU (different streams, or threads) race:
 * keep them on one stream, or use ebsp_zipline_batch with workspaces of your
 * own.  No kernel expects the array to be cleared; it keeps the last call's
 * contents.
 */
#define EBSP_STATIC_SCRATCH_BYTES (32u << 20)
size_t ebsp_zipline_static_scratch_bytes(void);
int ebsp_zipline_batch_static(const int64_t* ts, int64_t B, int32_t P, int32_t R,
                              int64_t* barrier, int32_t* iters, int64_t* wait,
                              int32_t* status, void* stream);

/*
 * The prediction folded in (Section III: a worker's iterations take similar
 * time, so its next R end timestamps are predicted from its most recent ones;
 * the paper gives no formula, the linear one is this library's reading):
 *
 *     t[p][i] = last_end[p] + (i + 1) * interval[p],   i = 0 .. R-1
 *
 * and then exactly the search of ebsp_zipline_batch over these rows, which are
 * never stored: the kernels compute them where they would have loaded them.
 *
 *   last_end  in  [B][P] int64, device: end timestamp of each worker's last
 *                 finished iteration (any fixed unit and epoch).
 *   interval  in  [B][P] int64, device: predicted iteration time, >= 0
 *                 (a negative one gives EBSP_STATUS_UNSORTED for the instance).
 *   workspace at least ebsp_predict_zipline_workspace_bytes(B, P, R) bytes;
 *   the other arguments, the status bits and the return codes: as for
 *   ebsp_zipline_batch.
 * Precondition: last_end + R * interval does not overflow int64.
 */
int ebsp_predict_zipline_batch(const int64_t* last_end, const int64_t* interval,
                               int64_t B, int32_t P, int32_t R,
                               int64_t* barrier, int32_t* iters, int64_t* wait,
                               int32_t* status, void* workspace, size_t workspace_bytes,
                               void* stream);

/*
 * A run of S supersteps (Fig. 1: a superstep is the time between two barriers;
 * Section III: the server decides barrier after barrier, each time from the
 * workers' most recent iteration times).  Superstep s predicts every worker's
 * next R end timestamps from the time it starts the superstep at and from its
 * iteration time in that superstep, searches them as
 * ebsp_predict_zipline_batch does, and lets all workers of the instance start
 * the next superstep together once the barrier and the synchronisation are
 * over:
 *
 *     start[0][b][p]  = last_end0[b][p]
 *     (barrier, iters, wait)[s][b] = search over start[s][b][p] + (i+1) * interval[s][b][p], i < R
 *     start[s+1][b][p] = barrier[s][b] + sync_cost           for every p
 *
 * The paper's training runs are not reproduced; this is the part of its
 * comparison that needs only iteration times: R = 1 is BSP with one iteration
 * per superstep (barrier = the slowest worker's end), larger R is ElasticBSP.
 * That workers run exactly as predicted within a superstep, that they all
 * resume at the same time and that a synchronisation takes a fixed time are
 * this library's readings (the paper states none of the three).
 *
 *   last_end0  in  [B][P] int64, device: each worker's start time of the run.
 *   interval   in  [S][B][P] int64, device: iteration time of worker p of
 *                  instance b during superstep s, >= 0.
 *   sync_cost      time from a barrier to the start of the next superstep, >= 0.
 *   barrier    out [S][B] int64; iters out [S][B][P] int32; wait out [S][B]
 *              int64; status out [S][B] int32 or NULL: per superstep as for
 *              ebsp_predict_zipline_batch.  An instance that raises a status
 *              bit in a superstep keeps its start times for the next one (when
 *              status is NULL this cannot be seen and its later results are
 *              undefined).
 *   workspace      at least ebsp_simulate_workspace_bytes(B, P, R) bytes (never
 *                  0 for a valid shape: it holds the start times), 256-byte
 *                  aligned.
 * The supersteps are enqueued one after the other on `stream`; nothing is
 * copied to the host in between.  S == 0 or B == 0 is a valid no-op.
 * Precondition: no start + R * interval overflows int64.  Return codes as above
 * (EBSP_ERR_SHAPE also for S < 0 or sync_cost < 0).
 */
size_t ebsp_simulate_workspace_bytes(int64_t B, int32_t P, int32_t R);
int ebsp_simulate_supersteps(const int64_t* last_end0, const int64_t* interval, int64_t sync_cost,
                             int64_t S, int64_t B, int32_t P, int32_t R,
                             int64_t* barrier, int32_t* iters, int64_t* wait, int32_t* status,
                             void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same search under the paper's formal objective (Section III "The
 * Problem": d_Z = max(Z) - min(Z), the waiting time of the fastest worker;
 * Section IV, Algorithm 2, which sweeps the merged timestamps with a set Z of
 * every worker's newest one; Fig. 3 caption for ties).  For a barrier c the
 * tightest Z holds every worker's latest timestamp <= c, so
 *
 *     dmin    = min_c ( c - min_p last_p(c) )   over timestamps c >= max_p t[p][0],
 *     barrier = the smallest c that attains it,
 *     iters[p]= #{ i : t[p][i] <= barrier }.
 *
 * Arguments, layouts, ownership and return codes as for ebsp_zipline_batch,
 * with dmin[B] (int64, device, >= 0) in place of wait[B] and a workspace of at
 * least ebsp_zipline_range_workspace_bytes() bytes.  No instance is refused
 * for its values: only EBSP_STATUS_UNSORTED can be raised (nothing is summed
 * over the workers, so there is no overflow precondition beyond max t - min t
 * fitting int64).
 */
size_t ebsp_zipline_range_workspace_bytes(int64_t B, int32_t P, int32_t R);
int ebsp_zipline_range_batch(const int64_t* ts, int64_t B, int32_t P, int32_t R,
                             int64_t* barrier, int32_t* iters, int64_t* dmin,
                             int32_t* status, void* workspace, size_t workspace_bytes,
                             void* stream);

/*
 * GridScan and FullGridScan, the paper's own comparators of the search (Section
 * IV: "GridScan", Algorithm 1, and the paragraph "FullGridScan"; Table I for
 * their cost, Table II for the comparison with ZipLine).  For a designated
 * point e of a designated row, Z holds e and every other row's point at the
 * shortest distance to e, and d_Z = max(Z) - min(Z) as in Section III.
 * full == 0 (GridScan): the row with the smallest first timestamp is
 * designated and the smallest d_Z over its R points is kept.  full != 0
 * (FullGridScan): every row is designated in turn (n*R sets).  Both are
 * heuristics for ebsp_zipline_range_batch's exact dmin: dz >= dmin always.
 *
 *   ts       in   [B][P][R] int64 device, every row non-decreasing; not modified
 *   barrier  out  [B] int64: max(Z*);  dz out [B] int64: d_Z* (>= 0)
 *   iters    out  [B][P] int32: 1 + the index in row p of the point Z* holds
 *   status   out  [B] int32 or NULL: EBSP_STATUS_UNSORTED if a row is not
 *                 non-decreasing (outputs then unspecified), else 0
 *   workspace     at least ebsp_gridscan_workspace_bytes(B, P, R, full) bytes,
 *                 256-byte aligned
 * Readings where the paper is silent: of two points of a row equally near to e
 * (and of equal timestamps) the earlier one is taken; of rows with the same
 * smallest first timestamp the first is designated; of equal d_Z the set met
 * first in (row, point) order is kept.  Precondition: max t - min t fits int64.
 * Asynchronous on `stream`, allocates nothing; return codes as above.
 */
size_t ebsp_gridscan_workspace_bytes(int64_t B, int32_t P, int32_t R, int32_t full);
int ebsp_gridscan_batch(const int64_t* ts, int64_t B, int32_t P, int32_t R, int32_t full,
                        int64_t* barrier, int32_t* iters, int64_t* dz, int32_t* status,
                        void* workspace, size_t workspace_bytes, void* stream);

/* Message for the last error returned on the calling thread (static,
 * thread-local storage; never NULL). */
const char* ebsp_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* EBSP_ZIPLINE_H */

/*
 * ebsp_zipline_bench.h -- benchmark and tuning hooks of libebsp_zipline.so.
 *
 * Not part of the search (ebsp_zipline.h): how a shape is handled, knobs that
 * change speed and never results, per-kernel timing, and plain streaming
 * kernels that serve as bandwidth yardsticks.  The knobs are process-wide
 * words read once at the start of every search call: set them before other
 * threads call into the library (a call that races with a change may see the
 * old or the new value of each word, and a workspace sized before a change may
 * be too small afterwards: the call then fails with EBSP_ERR_WORKSPACE).
 */
#ifndef EBSP_ZIPLINE_BENCH_H
#define EBSP_ZIPLINE_BENCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * How a shape is handled (for benchmarks' byte models; HOST array of 6):
 * info[0] = 1 if instances are cut into windows (0: one workgroup each),
 * info[1] = records per window workgroup, info[2] = fine bins per instance,
 * info[3] = upper bound of windows per instance, info[4] = entries a window
 * holds at most (all 0 when info[0] is 0); info[5] = slices per instance if
 * ebsp_zipline_batch searches stored rows of this shape with the frontier
 * sweep (0: it takes the path that info[0..4] describe).
 */
int ebsp_zipline_shape_info(int64_t B, int32_t P, int32_t R, int64_t* info);

/*
 * Tuning knobs (process-wide; call before ebsp_zipline_workspace_bytes, since
 * the workspace size depends on them; not thread-safe against running calls).
 *   window_cap  records one window workgroup holds on the multi-window path:
 *               4096, 8192 or 16384; 0 = chosen from P (the default).
 *   single_max  largest P*R that one workgroup handles whole (1..16384);
 *               0 = 16384 (the default).  Larger instances take the
 *               multi-window path.
 *   window_fill most entries of a window (at least 512); 0 = window_cap (the
 *               default: windows are packed as full as a workgroup can hold).
 * Results do not depend on any of them.  Returns EBSP_OK or EBSP_ERR_SHAPE.
 */
int ebsp_zipline_tune(int32_t window_cap, int32_t single_max, int32_t window_fill);

/*
 * Which stored-row batches ebsp_zipline_batch searches in one pass (the frontier
 * sweep) and how it slices them; process-wide, same rules as ebsp_zipline_tune.
 *   sweep_min   positive: instances of at least that many entries (P*R) and at
 *               most 1024 workers take the sweep; 0 = the default and negative:
 *               no batch does (every batch takes the kernels that predicted
 *               rows and the range objective use, which are faster today).
 *   slice_keys  entries per slice of an instance's value range (at least 256);
 *               0 = chosen from the batch.
 *   lines       128-byte lines of the input that one window of the sweep may
 *               ask for (at most 4096; raised to two per worker where it is
 *               less); 0 = chosen from P.
 * Results do not depend on any of them.  Returns EBSP_OK or EBSP_ERR_SHAPE.
 */
int ebsp_zipline_tune_sweep(int32_t sweep_min, int32_t slice_keys, int32_t lines);

/*
 * Per-kernel timing for benchmarks.  Between ebsp_zipline_profile_begin() and
 * ebsp_zipline_profile_end() every search call made by the calling thread
 * (any of the batch entry points; every superstep of ebsp_simulate_supersteps
 * counts as a call of its own) records a pair of HIP events around each kernel
 * it launches, on the call's own stream, without synchronising (events are
 * created up front, for at most max_calls calls; further calls run untimed).
 * Do not capture a stream into a HIP graph while a profile is open.
 * ebsp_zipline_profile_end() synchronises the device, writes to kernel_ms
 * (HOST array of ebsp_zipline_kernel_count() floats, may be NULL) the summed
 * duration in milliseconds of each kernel over the profiled calls and to
 * *calls (may be NULL) their number, and destroys the events.
 * These two calls allocate and free host memory and HIP events.
 */
int ebsp_zipline_profile_begin(int32_t max_calls);
int ebsp_zipline_profile_end(float* kernel_ms, int32_t* calls);

/*
 * Measurement yardstick, not part of the search: copies `bytes` (a positive
 * multiple of 16; both pointers 16-byte aligned device memory) from src to dst
 * with a plain streaming kernel on `stream`.  Benchmarks use it to see what
 * bandwidth, and what the HBM byte counters, read for a transfer of known size.
 * Counts as one call of an open profile.
 */
int ebsp_zipline_copy_probe(const void* src, void* dst, size_t bytes, void* stream);

/*
 * The same for kernels that mostly read: streams `bytes` (a positive multiple
 * of 16; src 16-byte aligned device memory) through a sum and adds the sums of
 * the workgroups' pieces to the EBSP_READ_SINK_WORDS words of sink (DEVICE,
 * 8-byte aligned; the caller sets them to zero if the values matter: together
 * they add up to the sum of all 32-bit words read).  Counts as one call of an
 * open profile.
 */
#define EBSP_READ_SINK_WORDS 256
int ebsp_zipline_read_probe(const void* src, size_t bytes, uint64_t* sink, void* stream);

/*
 * What the current device reports of its memory (HOST pointers): the memory
 * clock in kHz and the bus width in bits, as hipDeviceGetAttribute gives them.
 * With double data rate the peak they imply is 2 * clock * bus / 8 bytes/s.
 */
int ebsp_zipline_memory_info(int32_t* clock_khz, int32_t* bus_bits);

/* Number of distinct kernels the library may launch, and their names
 * (static storage; NULL if i is out of range). */
int         ebsp_zipline_kernel_count(void);
const char* ebsp_zipline_kernel_name(int i);

#ifdef __cplusplus
}
#endif
#endif /* EBSP_ZIPLINE_BENCH_H */

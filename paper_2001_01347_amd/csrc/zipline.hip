// ZipLine barrier search for MI355X (gfx950, wave64).
//
// Implements the C ABI declared in include/ebsp_zipline.h.  The search is the
// sweep of Algorithm 2 of the ElasticBSP paper (arXiv 2001.01347) with the
// summed waiting time as objective (Section III; Fig. 1 caption), recast for
// a GPU:
//
//   * the set Z of Algorithm 2 (newest timestamp per worker) is never built.
//     With delta[p][i] = t[p][i] - t[p][i-1], the sum of the elements of Z
//     after the sweep has passed timestamp c is the prefix sum of the deltas
//     of all elements <= c in sorted order, so
//         wait(c) = P*c - prefix(c)
//     and the sweep becomes sort -> scan -> arg-min;
//   * every row of the input is already sorted (rows are iteration sequences,
//     Section III), so the merged set Omega can be cut into windows of
//     consecutive values without moving any data: a window takes one
//     contiguous segment of every row.  A window that fits in LDS is searched
//     by one workgroup, and the value of the prefix at the window start is
//     known from the row elements just before the segments, so windows need
//     no carry from one another;
//   * inside a window the sort is a counting sort into value buckets, exact
//     bounds per bucket drop the buckets that cannot hold the minimum, and
//     only the entries of the remaining buckets are ordered and evaluated;
//   * small instances (P*R <= 16384) are one window: one workgroup each, no
//     scratch memory, one kernel.
//
// Device code, by header (each includes the one before it):
//   zl_common.h    types, records, wave/block primitives, the fine-bin map
//   zl_rows.h      rows of an instance (stored or predicted), zl_iters
//   zl_sort.h      general search of a window: radix sort, scan, arg-min
//   zl_bucket.h    fast search of a window: buckets, bounds, evaluation
//   zl_gather.h    zl_delta: row segments -> (key, delta) records in registers
//   zl_walk.h      general search of a value interval of any size
//   zl_instance.h  one workgroup per instance
//   zl_plan.h      zl_bounds, zl_partition, zl_bincount, zl_plan (the windows)
//   zl_window.h    window kernels of the summed-wait search
//   zl_range.h     the objective max(Z) - min(Z)
//   zl_finish.h    reduction over windows, zl_iters; the copy yardstick
//   zl_sweep.h     the frontier sweep: stored rows searched in one pass, no crossing table
//   zl_gridscan.h  GridScan and FullGridScan, the paper's comparators
// This file: the host side (plans, launches, the C entry points).
#include <hip/hip_runtime.h>
#include <atomic>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "ebsp_zipline.h"
#include "ebsp_zipline_bench.h"
#include "zl_gridscan.h"    // pulls in the other device headers, in dependency order

namespace {

// ---------------------------------------------------------------------------
// Host side.

thread_local char g_err[256] = "";

int fail(int code, const char* msg)
{
    snprintf(g_err, sizeof g_err, "%s", msg);
    return code;
}

// The kernels are built for gfx950 only: refuse any other device by name instead of
// letting a launch fail.  Asked once per device; the answer is kept.
int check_device()
{
    constexpr int KNOWN = 64;
    static std::atomic<signed char> seen[KNOWN];       // 0: not asked yet, 1: gfx950, -1: something else
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return fail(EBSP_ERR_DEVICE, "no current HIP device");
    signed char state = dev >= 0 && dev < KNOWN ? seen[dev].load(std::memory_order_relaxed) : 0;
    if (state == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return fail(EBSP_ERR_DEVICE, "hipGetDeviceProperties failed");
        state = strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? 1 : -1;
        if (dev >= 0 && dev < KNOWN) seen[dev].store(state, std::memory_order_relaxed);
    }
    if (state < 0) return fail(EBSP_ERR_DEVICE, "the current device is not a gfx950 (MI355X): this library has code for nothing else");
    return EBSP_OK;
}

enum KernelId { K_INSTANCE = 0, K_INSTANCE_GENERAL, K_BOUNDS, K_PARTITION, K_BINCOUNT, K_PLAN, K_WINDOW,
                K_WINDOW_GENERAL, K_FINISH, K_COPY, K_RANGE_INSTANCE, K_RANGE_WINDOW, K_PARTITION_PRED, K_RANGE_FAST, K_ADVANCE, K_SWEEP, K_SWEEP_FINISH, K_GRIDSCAN, K_GRIDSCAN_FINISH, K_READ, K_INSTANCE_REG, K_COUNT };
const char* const kKernelNames[K_COUNT] = {
    "zl_instance_kernel", "zl_instance_general_kernel", "zl_bounds_kernel", "zl_partition_kernel",
    "zl_bincount_kernel", "zl_plan_kernel", "zl_window_kernel", "zl_window_general_kernel",
    "zl_finish_kernel", "zl_copy_kernel", "zl_range_instance_kernel", "zl_range_window_kernel",
    "zl_partition_pred_kernel", "zl_range_fast_kernel", "zl_advance_kernel", "zl_sweep_kernel", "zl_sweep_finish_kernel", "zl_gridscan_kernel",
    "zl_gridscan_finish_kernel", "zl_read_kernel", "zl_instance_reg_kernel"};

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Shape-dependent sizes of the multi-window path.
struct Tuning {          // 0: choose by shape
    int window_cap;
    int single_max;
    int window_fill;
    int sweep_min;       // smallest P*R that takes the frontier sweep (0: the default, < 0: never)
    int slice_keys;      // entries per slice of the sweep (0: chosen from the batch)
    int sweep_lines;     // lines of a plan of the sweep (0: chosen from P)
};
// Set before any thread calls a search (the header says so); read once per call, word by word.
std::atomic<int> g_tune_window_cap{0}, g_tune_single_max{0}, g_tune_window_fill{0}, g_tune_sweep_min{0}, g_tune_slice_keys{0}, g_tune_sweep_lines{0};
Tuning tuning()
{
    Tuning t;
    t.window_cap = g_tune_window_cap.load(std::memory_order_relaxed);
    t.single_max = g_tune_single_max.load(std::memory_order_relaxed);
    t.window_fill = g_tune_window_fill.load(std::memory_order_relaxed);
    t.sweep_min = g_tune_sweep_min.load(std::memory_order_relaxed);
    t.slice_keys = g_tune_slice_keys.load(std::memory_order_relaxed);
    t.sweep_lines = g_tune_sweep_lines.load(std::memory_order_relaxed);
    return t;
}

// The frontier sweep (zl_sweep.h) takes stored rows of these shapes under the summed-wait objective.
constexpr int SWEEP_NT = 512, SWEEP_LINES = 4096, SWEEP_BUCKETS = 4096, SWEEP_LIST = 2048;
constexpr int SWEEP_DEFAULT_ON = 1;              // 0: the sweep is the default for its shapes; 1: only where ebsp_zipline_tune_sweep asks for it
constexpr int SWEEP_MIN_DEFAULT = 8192;          // instances of fewer entries: one workgroup of zl_instance_kernel each
constexpr int SWEEP_PMAX = 1024;                 // every row with entries left needs a line of its own and one to spare

struct Plan {
    bool sweep;        // stored rows go through the frontier sweep
    int nslices;       // slices per instance there
    int lines;         // lines of a plan there
    size_t off_spartial, off_best, sweep_bytes;
    bool multi;
    int cap;           // records per window workgroup
    int fill;          // most entries of a window (unless a single fine bin holds more)
    int part_stored, part_pred;   // groups of rows whose column sums the partition kernels write (stored / predicted rows)
    int bins;          // fine bins per instance
    int stride;        // bins + 1 crossing indices per row
    int max_win;       // windows per instance <= max_win
    bool narrow;       // crossing indices fit 16 bits
    size_t off_info, off_seg, off_cross, off_part, off_below, off_winstart, off_winval, off_partial, off_rowpar, off_wide, bytes;
};

// single_limit: the most entries one workgroup takes whole on the path the plan is for;
// list_room: windows leave a quarter or more of the workgroup's records free (the fast range search keeps its short list there)
bool make_plan(i64 B, int P, int R, Plan& pl, int single_limit = SINGLE_MAX, bool list_room = false, bool stored_sum = false)
{
    if (B < 0 || P < 1 || R < 1) return false;
    const i64 n = (i64)P * (i64)R;
    if (n >= (1ll << 31)) return false;
    memset(&pl, 0, sizeof pl);
    const Tuning g_tune = tuning();
    {
        const i64 sweep_min = g_tune.sweep_min > 0 ? g_tune.sweep_min : SWEEP_MIN_DEFAULT;
        pl.sweep = stored_sum && g_tune.sweep_min >= SWEEP_DEFAULT_ON && n >= sweep_min && n < (1ll << 29) && P <= SWEEP_PMAX && B > 0;
        if (pl.sweep) {
            // about 2048 slices per batch (four rounds of two workgroups per CU), each long enough to pay for the
            // searches that open it (64 entries per row or more) and short enough to spread an instance over the chip
            i64 keys = g_tune.slice_keys > 0 ? g_tune.slice_keys : B * n / 2048;
            if (g_tune.slice_keys <= 0) {
                if (keys < 32768) keys = 32768;
                if (keys > 262144) keys = 262144;
                if (keys < 64ll * P) keys = 64ll * P;
            }
            i64 ns = (n + keys - 1) / keys;
            if (ns > 4096) ns = 4096;
            pl.nslices = (int)(ns < 1 ? 1 : ns);
            // four lines a row: a window then takes about forty entries of every row, most of what is loaded
            int lines = g_tune.sweep_lines > 0 ? g_tune.sweep_lines : 4 * P;
            lines = (lines + 31) / 32 * 32;
            if (lines < 2 * P) lines = (2 * P + 31) / 32 * 32;
            if (lines < 128) lines = 128;
            if (lines > SWEEP_LINES) lines = SWEEP_LINES;
            pl.lines = lines;
            size_t o = 0;                                       // (the first two as in the other layout below)
            pl.off_info = o;     o = align_up(o + (size_t)B * sizeof(InstInfo), 256);
            pl.off_seg = o;      o = align_up(o + (size_t)B * SEGS * sizeof(SegEntry), 256);
            pl.off_spartial = o; o = align_up(o + (size_t)B * pl.nslices * sizeof(Partial), 256);
            pl.off_best = o;     o = align_up(o + (size_t)B * sizeof(i64), 256);
            pl.sweep_bytes = o;
        }
    }
    int single_max = g_tune.single_max > 0 ? g_tune.single_max : SINGLE_MAX;
    if (single_max > single_limit) single_max = single_limit;
    pl.multi = n > single_max;
    if (!pl.multi) return true;
    // the per-window cost has a term proportional to P: larger windows for more rows
    pl.cap = g_tune.window_cap > 0 ? g_tune.window_cap : (P >= 1536 ? 16384 : (P >= 512 ? 8192 : 4096));
    const int fine_shift = (pl.cap == 16384 ? 14 : (pl.cap == 8192 ? 13 : 12)) - 3;       // fine bins of cap/8 keys on average
    pl.fill = g_tune.window_fill > 0 && g_tune.window_fill < pl.cap ? g_tune.window_fill : pl.cap;
    if (list_room) {
        // with few workers a larger share of a window's entries is min(Z) at some time and has to be listed
        const int room = P < 128 ? pl.cap / 2 : pl.cap / 4;
        if (pl.fill > pl.cap - room) pl.fill = pl.cap - room;
    }
    pl.bins = (int)((n + (1 << fine_shift) - 1) >> fine_shift);
    pl.stride = (pl.bins + 1 + 7) / 8 * 8;              // rows of cross start on 16-byte boundaries
    // two windows in a row hold more than `fill` keys, or they would be one; a whole number of workgroups per instance
    pl.max_win = (int)((2 * n / pl.fill + 3 + WINDOWS_PER_BLOCK - 1) / WINDOWS_PER_BLOCK * WINDOWS_PER_BLOCK);
    size_t o = 0;
    pl.off_info = o;     o = align_up(o + (size_t)B * sizeof(InstInfo), 256);
    pl.off_seg = o;      o = align_up(o + (size_t)B * SEGS * sizeof(SegEntry), 256);
    pl.narrow = R < 65536;
    pl.off_cross = o;    o = align_up(o + (size_t)B * P * pl.stride * (pl.narrow ? 2 : 4), 256);
    pl.part_stored = pl.stride <= PART_MAX_STRIDE ? (P + PART_ROWS - 1) / PART_ROWS : 0;     // 0: zl_bincount reads cross itself
    pl.part_pred = (P + PRED_ROWS_PER_BLOCK - 1) / PRED_ROWS_PER_BLOCK;
    const int part_rows = pl.part_stored > pl.part_pred ? pl.part_stored : pl.part_pred;
    pl.off_part = o;     o = align_up(o + (size_t)B * part_rows * pl.stride * sizeof(u32), 256);
    pl.off_below = o;    o = align_up(o + (size_t)B * pl.stride * sizeof(u32), 256);
    pl.off_winstart = o; o = align_up(o + (size_t)B * (pl.max_win + 1) * sizeof(u32), 256);
    pl.off_winval = o;   o = align_up(o + (size_t)B * pl.max_win * sizeof(WinVal), 256);
    pl.off_partial = o;  o = align_up(o + (size_t)B * pl.max_win * sizeof(Partial), 256);
    pl.off_rowpar = o;   o = align_up(o + (size_t)B * P * sizeof(uint2), 256);      // predicted rows only
    pl.off_wide = o;     o = align_up(o + (size_t)B * WIDE_MARKS * sizeof(u32), 256);
    pl.bytes = o;
    return true;
}

// Optional per-kernel timing: while a profile is open on this thread every
// launch is bracketed by two events taken from a pool created up front.
struct Profile {
    bool on = false;
    int max_calls = 0, calls = 0;
    hipEvent_t* ev = nullptr;      // [max_calls][K_COUNT][2]
    bool* used = nullptr;          // [max_calls][K_COUNT]
};
thread_local Profile g_prof;

hipEvent_t* prof_slot(int kid, int which)
{
    if (!g_prof.on || g_prof.calls >= g_prof.max_calls) return nullptr;
    if (which == 0) g_prof.used[g_prof.calls * K_COUNT + kid] = true;
    return &g_prof.ev[(g_prof.calls * K_COUNT + kid) * 2 + which];
}

#define LAUNCH(kid, kernel, grid, block, ...)                                              \
    do {                                                                                   \
        if (hipEvent_t* e0_ = prof_slot(kid, 0)) (void)hipEventRecord(*e0_, st);           \
        hipLaunchKernelGGL(kernel, grid, block, 0, st, __VA_ARGS__);                       \
        if (hipEvent_t* e1_ = prof_slot(kid, 1)) (void)hipEventRecord(*e1_, st);           \
        hipError_t e_ = hipGetLastError();                                                 \
        if (e_ != hipSuccess) {                                                            \
            snprintf(g_err, sizeof g_err, "%s: %s", kKernelNames[kid], hipGetErrorString(e_)); \
            return EBSP_ERR_LAUNCH;                                                        \
        }                                                                                  \
    } while (0)

// The front of the multi-window path, shared by the objectives: per-instance facts and
// fine-bin map, crossing indices, exact bin counts, windows.
int plan_windows(const Plan& pl, const i64* ts, const i64* le, const i64* iv, i64 B, int P, int R,
                 char* wsp, int* status, bool summed, hipStream_t st)
{
    const bool pred = ts == nullptr;
    InstInfo* info = (InstInfo*)(wsp + pl.off_info);
    SegEntry* segtab = (SegEntry*)(wsp + pl.off_seg);
    void* cross = (void*)(wsp + pl.off_cross);
    u32* part = (u32*)(wsp + pl.off_part);
    u32* below = (u32*)(wsp + pl.off_below);
    u32* winstart = (u32*)(wsp + pl.off_winstart);
    WinVal* winval = (WinVal*)(wsp + pl.off_winval);
    uint2* rowpar = pred ? (uint2*)(wsp + pl.off_rowpar) : nullptr;
    u32* widebin = (u32*)(wsp + pl.off_wide);
    const i64 nrows = B * (i64)P;
    const i64 kblocks = (pl.stride + 255) / 256;
    const i64 widest = pl.part_stored > pl.part_pred ? pl.part_stored : pl.part_pred;
    if (kblocks * B > 0x7fffffffll || widest * B > 0x7fffffffll) return fail(EBSP_ERR_SHAPE, "batch too large for one call");
    LAUNCH(K_BOUNDS, (zl_bounds_kernel<256>), dim3((unsigned)B), dim3(256), ts, le, iv, P, R, pl.bins, info, segtab, rowpar, status, summed,
           (i64*)nullptr);
    int part_rows;                                    // rows of partial column sums per instance (0: none, count from cross)
    if (pred) {
        part_rows = pl.part_pred;
        // two bins per thread where an instance's bins still make many workgroups
#define LAUNCH_PARTITION_PRED(CT_, KPT_)                                                                         \
    LAUNCH(K_PARTITION_PRED, (zl_partition_pred_kernel<CT_, KPT_>),                                              \
           dim3((unsigned)((pl.stride + 256 * KPT_ - 1) / (256 * KPT_) * B), (unsigned)part_rows), dim3(256),     \
           le, iv, P, R, info, segtab, (CT_*)cross, pl.stride, part)
        if (pl.stride >= 2048) {
            if (pl.narrow) LAUNCH_PARTITION_PRED(unsigned short, 2); else LAUNCH_PARTITION_PRED(u32, 2);
        } else {
            if (pl.narrow) LAUNCH_PARTITION_PRED(unsigned short, 1); else LAUNCH_PARTITION_PRED(u32, 1);
        }
#undef LAUNCH_PARTITION_PRED
    } else if (pl.part_stored > 0) {
        part_rows = pl.part_stored;
        if (pl.narrow)
            LAUNCH(K_PARTITION, zl_partition_sum_kernel<unsigned short>, dim3((unsigned)(B * part_rows)), dim3(PART_ROWS * WAVE),
                   ts, P, R, part_rows, info, widebin, segtab, (unsigned short*)cross, pl.stride, part, status);
        else
            LAUNCH(K_PARTITION, zl_partition_sum_kernel<u32>, dim3((unsigned)(B * part_rows)), dim3(PART_ROWS * WAVE),
                   ts, P, R, part_rows, info, widebin, segtab, (u32*)cross, pl.stride, part, status);
    } else {
        part_rows = 0;
        if (pl.narrow)
            LAUNCH(K_PARTITION, (zl_partition_kernel<256, unsigned short>), dim3((unsigned)((nrows + 3) / 4)), dim3(256),
                   ts, nrows, P, R, info, widebin, segtab, (unsigned short*)cross, pl.stride, status);
        else
            LAUNCH(K_PARTITION, (zl_partition_kernel<256, u32>), dim3((unsigned)((nrows + 3) / 4)), dim3(256),
                   ts, nrows, P, R, info, widebin, segtab, (u32*)cross, pl.stride, status);
    }
    if (part_rows > 0)        // the partial sums are exact counts already: nothing to clamp
        LAUNCH(K_BINCOUNT, zl_bincount_kernel<u32>, dim3((unsigned)(kblocks * B)), dim3(256),
               (const u32*)part, part_rows, 0x7fffffff, pl.stride, info, below);
    else if (pl.narrow)
        LAUNCH(K_BINCOUNT, zl_bincount_kernel<unsigned short>, dim3((unsigned)(kblocks * B)), dim3(256),
               (const unsigned short*)cross, P, R, pl.stride, info, below);
    else
        LAUNCH(K_BINCOUNT, zl_bincount_kernel<u32>, dim3((unsigned)(kblocks * B)), dim3(256),
               (const u32*)cross, P, R, pl.stride, info, below);
    if (pl.bins <= 1024)      // small instances, many of them: small workgroups
        LAUNCH(K_PLAN, (zl_plan_kernel<256, 1024>), dim3((unsigned)B), dim3(256), info, segtab, below, pl.stride, widebin, pred, winstart, winval,
               pl.max_win, (u32)pl.fill, (u32)(pl.cap / 8));
    else
        LAUNCH(K_PLAN, (zl_plan_kernel<1024, 4096>), dim3((unsigned)B), dim3(1024), info, segtab, below, pl.stride, widebin, pred, winstart, winval,
               pl.max_win, (u32)pl.fill, (u32)(pl.cap / 8));
    return EBSP_OK;
}

// The rows are either stored (ts != nullptr) or predicted: t[p][i] = le[p] + (i + 1) * iv[p] (ts == nullptr).
int run_batch(const i64* ts, const i64* le, const i64* iv, i64 B, int P, int R,
              i64* barrier, int* iters, i64* wait, int* status,
              void* workspace, size_t workspace_bytes, hipStream_t st)
{
    Plan pl;
    const bool pred = ts == nullptr;
    if (!make_plan(B, P, R, pl, SINGLE_MAX, false, !pred)) return fail(EBSP_ERR_SHAPE, "invalid shape: need B >= 0, P >= 1, R >= 1, P*R < 2^31");
    if (B == 0) return EBSP_OK;
    if ((pred && (!le || !iv)) || !barrier || !iters || !wait)
        return fail(EBSP_ERR_NULL, "the input arrays, barrier, iters and wait must not be NULL");
    if (B > 0x7fffffffll) return fail(EBSP_ERR_SHAPE, "B must be below 2^31");
    const int n = P * R;

    if (pl.sweep) {
        // stored rows in one pass: instance facts and slices, the sweep, the reduction over slices with zl_iters
        if (!workspace) return fail(EBSP_ERR_NULL, "this shape needs a workspace");
        if (workspace_bytes < pl.sweep_bytes) return fail(EBSP_ERR_WORKSPACE, "workspace smaller than ebsp_zipline_workspace_bytes()");
        if (((uintptr_t)workspace & 255u) != 0) return fail(EBSP_ERR_WORKSPACE, "workspace must be 256-byte aligned");
        const i64 pblocks = (P + 255) / 256;
        if (B * (i64)pl.nslices > 0x7fffffffll || pblocks * B > 0x7fffffffll) return fail(EBSP_ERR_SHAPE, "batch too large for one call");
        if (int rc = check_device()) return rc;
        char* wsp = (char*)workspace;
        InstInfo* info = (InstInfo*)(wsp + pl.off_info);
        SegEntry* segtab = (SegEntry*)(wsp + pl.off_seg);
        Partial* spartial = (Partial*)(wsp + pl.off_spartial);
        i64* best = (i64*)(wsp + pl.off_best);
        LAUNCH(K_BOUNDS, (zl_bounds_kernel<256>), dim3((unsigned)B), dim3(256), ts, le, iv, P, R, pl.nslices, info, segtab,
               (uint2*)nullptr, status, true, best);
        const dim3 sgrid((unsigned)(B * (i64)pl.nslices));
        LAUNCH(K_SWEEP, (zl_sweep_kernel<SWEEP_NT, SWEEP_LINES, SWEEP_BUCKETS, SWEEP_LIST, SWEEP_PMAX>), sgrid, dim3(SWEEP_NT),
               ts, B, P, R, pl.nslices, pl.lines, info, segtab, best, spartial, status);
        LAUNCH(K_SWEEP_FINISH, (zl_sweep_finish_kernel<256>), dim3((unsigned)(pblocks * B)), dim3(256),
               ts, P, R, pl.nslices, info, spartial, barrier, iters, wait);
        return EBSP_OK;
    }

    if (!pl.multi) {
        if (int rc = check_device()) return rc;
        const int rshift = (R & (R - 1)) == 0 ? __builtin_ctz((unsigned)R) : -1;
        const dim3 grid((unsigned)B);
#define LAUNCH_INSTANCE(NT_, ITEMS_)                                                                        \
    do {                                                                                                    \
        if (pred) LAUNCH(K_INSTANCE, (zl_instance_kernel<NT_, ITEMS_, true>), grid, dim3(NT_), ts, le, iv, P, R, rshift, \
                         barrier, iters, wait, status);                                                     \
        else LAUNCH(K_INSTANCE, (zl_instance_kernel<NT_, ITEMS_, false>), grid, dim3(NT_), ts, le, iv, P, R, rshift, \
                    barrier, iters, wait, status);                                                          \
    } while (0)
        // larger instances keep their records in registers: less LDS, several workgroups per CU
#define LAUNCH_INSTANCE_REG(NT_, ITEMS_)                                                                    \
    do {                                                                                                    \
        if (pred) LAUNCH(K_INSTANCE_REG, (zl_instance_reg_kernel<NT_, ITEMS_, true>), grid, dim3(NT_), ts, le, iv, P, R, rshift, \
                         barrier, iters, wait, status);                                                     \
        else LAUNCH(K_INSTANCE_REG, (zl_instance_reg_kernel<NT_, ITEMS_, false>), grid, dim3(NT_), ts, le, iv, P, R, rshift, \
                    barrier, iters, wait, status);                                                          \
    } while (0)
        if (n <= 256) LAUNCH_INSTANCE(128, 2);
        else if (n <= 1024) LAUNCH_INSTANCE(256, 4);       // (batches of so small instances are often small too: the shorter chain per thread wins)
        else if (n <= 2048) LAUNCH_INSTANCE_REG(256, 8);
        else if (n <= 4096) LAUNCH_INSTANCE_REG(256, 16);
        else if (n <= 8192) LAUNCH_INSTANCE_REG(512, 16);
        else LAUNCH_INSTANCE_REG(1024, 16);
#undef LAUNCH_INSTANCE_REG
#undef LAUNCH_INSTANCE
        // what the kernel above left: the general search in the smallest workgroup whose records hold an
        // instance (half of NT * ITEMS with 64-bit deltas), as many workgroups as fit the chip at once
#define LAUNCH_GENERAL(NT_, ITEMS_, PER_CU_)                                                                 \
    LAUNCH(K_INSTANCE_GENERAL, (zl_instance_general_kernel<NT_, ITEMS_>),                                    \
           dim3((unsigned)(B < PER_CU_ * GENERAL_GRID ? B : PER_CU_ * GENERAL_GRID)), dim3(NT_),            \
           ts, le, iv, B, P, R, barrier, iters, wait, status)
        if (n <= 1024) LAUNCH_GENERAL(256, 8, 7);
        else if (n <= 2048) LAUNCH_GENERAL(256, 16, 4);
        else if (n <= 4096) LAUNCH_GENERAL(512, 16, 2);
        else LAUNCH_GENERAL(LARGE_NT, LARGE_ITEMS, 1);
#undef LAUNCH_GENERAL
        return EBSP_OK;
    }

    if (!workspace) return fail(EBSP_ERR_NULL, "this shape needs a workspace");
    if (workspace_bytes < pl.bytes) return fail(EBSP_ERR_WORKSPACE, "workspace smaller than ebsp_zipline_workspace_bytes()");
    if (((uintptr_t)workspace & 255u) != 0) return fail(EBSP_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    const i64 total_win = B * (i64)pl.max_win;
    if (total_win + 8 > 0x7fffffffll || B * (i64)P > (0x7fffffffll * 4)) return fail(EBSP_ERR_SHAPE, "batch too large for one call");

    char* wsp = (char*)workspace;
    InstInfo* info = (InstInfo*)(wsp + pl.off_info);
    void* cross = (void*)(wsp + pl.off_cross);
    u32* winstart = (u32*)(wsp + pl.off_winstart);
    WinVal* winval = (WinVal*)(wsp + pl.off_winval);
    Partial* partial = (Partial*)(wsp + pl.off_partial);
    uint2* rowpar = pred ? (uint2*)(wsp + pl.off_rowpar) : nullptr;

    const i64 pblocks = (P + 255) / 256;
    if (pblocks * B > 0x7fffffffll) return fail(EBSP_ERR_SHAPE, "batch too large for one call");
    if (int rc = check_device()) return rc;
    if (int rc = plan_windows(pl, ts, le, iv, B, P, R, wsp, status, true, st)) return rc;
    const u32 groups = (u32)(pl.max_win / WINDOWS_PER_BLOCK);
    const u32 groups_inv = groups > 1 ? (u32)((1ull << 32) / groups) : 0xffffffffu;
    const unsigned wgrid = (unsigned)((B * (i64)groups + 7) / 8 * 8);
#define LAUNCH_WINDOW(NT_, CT_)                                                                              \
    do {                                                                                                     \
        if (pred) LAUNCH(K_WINDOW, (zl_window_kernel<NT_, 16, CT_, true>), dim3(wgrid), dim3(NT_), ts, rowpar, B, P, R, info, \
                         (const CT_*)cross, pl.stride, winstart, winval, pl.max_win, groups, groups_inv, partial); \
        else LAUNCH(K_WINDOW, (zl_window_kernel<NT_, 16, CT_, false>), dim3(wgrid), dim3(NT_), ts, rowpar, B, P, R, info, \
                    (const CT_*)cross, pl.stride, winstart, winval, pl.max_win, groups, groups_inv, partial);  \
    } while (0)
    if (pl.cap == 16384) {
        if (pl.narrow) LAUNCH_WINDOW(1024, unsigned short); else LAUNCH_WINDOW(1024, u32);
    } else if (pl.cap == 8192) {
        if (pl.narrow) LAUNCH_WINDOW(512, unsigned short); else LAUNCH_WINDOW(512, u32);
    } else {
        if (pl.narrow) LAUNCH_WINDOW(256, unsigned short); else LAUNCH_WINDOW(256, u32);
    }
#undef LAUNCH_WINDOW
    if (pl.cap <= 4096)       // such windows fit a 512-thread workgroup's general search: two workgroups per CU
        LAUNCH(K_WINDOW_GENERAL, (zl_window_general_kernel<512, 16>),
               dim3((unsigned)(total_win < 2 * GENERAL_GRID ? total_win : 2 * GENERAL_GRID)), dim3(512),
               ts, le, iv, B, P, R, info, cross, pl.narrow, pl.stride, winstart, winval, pl.max_win, partial, status);
    else
        LAUNCH(K_WINDOW_GENERAL, (zl_window_general_kernel<LARGE_NT, LARGE_ITEMS>),
               dim3((unsigned)(total_win < GENERAL_GRID ? total_win : GENERAL_GRID)), dim3(LARGE_NT),
               ts, le, iv, B, P, R, info, cross, pl.narrow, pl.stride, winstart, winval, pl.max_win, partial, status);
    LAUNCH(K_FINISH, (zl_finish_kernel<256>), dim3((unsigned)(pblocks * B)), dim3(256),
           ts, le, iv, P, R, info, (const SegEntry*)(wsp + pl.off_seg), (const void*)cross, pl.narrow, pl.stride,
           partial, pl.max_win, barrier, iters, wait);
    return EBSP_OK;
}

// The search under the paper's formal objective; the multi-window path shares the
// kernels that cut an instance into windows.
constexpr int RANGE_SINGLE_MAX = WinCfg<LARGE_NT, LARGE_ITEMS>::CAP_WIDE;


int run_range_batch(const i64* ts, i64 B, int P, int R, i64* barrier, int* iters, i64* dmin, int* status,
                    void* workspace, size_t workspace_bytes, hipStream_t st)
{
    Plan pl;
    if (!make_plan(B, P, R, pl, RANGE_SINGLE_MAX, true))
        return fail(EBSP_ERR_SHAPE, "invalid shape: need B >= 0, P >= 1, R >= 1, P*R < 2^31");
    if (B == 0) return EBSP_OK;
    if (!ts || !barrier || !iters || !dmin) return fail(EBSP_ERR_NULL, "ts, barrier, iters and dmin must not be NULL");
    if (B > 0x7fffffffll) return fail(EBSP_ERR_SHAPE, "B must be below 2^31");
    if (!pl.multi) {
        if (int rc = check_device()) return rc;
        // the smallest workgroup whose records hold the instance (half of NT * ITEMS in the 12-byte form):
        // several small instances share a CU
        const i64 n = (i64)P * R;
        if (n <= 1024)
            LAUNCH(K_RANGE_INSTANCE, (zl_range_instance_kernel<256, 8>), dim3((unsigned)B), dim3(256),
                   ts, P, R, barrier, iters, dmin, status);
        else if (n <= 2048)
            LAUNCH(K_RANGE_INSTANCE, (zl_range_instance_kernel<256, 16>), dim3((unsigned)B), dim3(256),
                   ts, P, R, barrier, iters, dmin, status);
        else if (n <= 4096)
            LAUNCH(K_RANGE_INSTANCE, (zl_range_instance_kernel<512, 16>), dim3((unsigned)B), dim3(512),
                   ts, P, R, barrier, iters, dmin, status);
        else
            LAUNCH(K_RANGE_INSTANCE, (zl_range_instance_kernel<LARGE_NT, LARGE_ITEMS>), dim3((unsigned)B), dim3(LARGE_NT),
                   ts, P, R, barrier, iters, dmin, status);
        return EBSP_OK;
    }
    if (!workspace) return fail(EBSP_ERR_NULL, "this shape needs a workspace");
    if (workspace_bytes < pl.bytes) return fail(EBSP_ERR_WORKSPACE, "workspace smaller than ebsp_zipline_range_workspace_bytes()");
    if (((uintptr_t)workspace & 255u) != 0) return fail(EBSP_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    const i64 total_win = B * (i64)pl.max_win;
    if (total_win + 8 > 0x7fffffffll || B * (i64)P > (0x7fffffffll * 4)) return fail(EBSP_ERR_SHAPE, "batch too large for one call");

    char* wsp = (char*)workspace;
    InstInfo* info = (InstInfo*)(wsp + pl.off_info);
    void* cross = (void*)(wsp + pl.off_cross);
    u32* winstart = (u32*)(wsp + pl.off_winstart);
    WinVal* winval = (WinVal*)(wsp + pl.off_winval);
    Partial* partial = (Partial*)(wsp + pl.off_partial);

    const i64 pblocks = (P + 255) / 256;
    if (pblocks * B > 0x7fffffffll) return fail(EBSP_ERR_SHAPE, "batch too large for one call");
    if (int rc = check_device()) return rc;
    if (int rc = plan_windows(pl, ts, nullptr, nullptr, B, P, R, wsp, status, false, st)) return rc;
    const u32 groups = (u32)(pl.max_win / WINDOWS_PER_BLOCK);
    const u32 groups_inv = groups > 1 ? (u32)((1ull << 32) / groups) : 0xffffffffu;
    const unsigned wgrid = (unsigned)((B * (i64)groups + 7) / 8 * 8);
#define LAUNCH_RANGE(NT_, CT_)                                                                               \
    LAUNCH(K_RANGE_FAST, (zl_range_fast_kernel<NT_, 16, CT_>), dim3(wgrid), dim3(NT_), ts, B, P, R, info,   \
           (const CT_*)cross, pl.stride, winstart, winval, pl.max_win, groups, groups_inv, partial)
    if (pl.cap == 16384) {
        if (pl.narrow) LAUNCH_RANGE(1024, unsigned short); else LAUNCH_RANGE(1024, u32);
    } else if (pl.cap == 8192) {
        if (pl.narrow) LAUNCH_RANGE(512, unsigned short); else LAUNCH_RANGE(512, u32);
    } else {
        if (pl.narrow) LAUNCH_RANGE(256, unsigned short); else LAUNCH_RANGE(256, u32);
    }
#undef LAUNCH_RANGE
    // what the fast kernel left: the sort-based search, one workgroup per marked window
    // the windows the fast kernel marked; more workgroups than fit at once, so that uneven shares even out
    if (pl.cap <= 4096)       // such windows fit a 512-thread workgroup's sort (three workgroups per CU)
        LAUNCH(K_RANGE_WINDOW, (zl_range_window_kernel<512, 16>), dim3(8 * GENERAL_GRID), dim3(512),
               ts, B, P, R, info, cross, pl.narrow, pl.stride, winstart, winval, pl.max_win, partial, status);
    else
        LAUNCH(K_RANGE_WINDOW, (zl_range_window_kernel<LARGE_NT, LARGE_ITEMS>), dim3(4 * GENERAL_GRID), dim3(LARGE_NT),
               ts, B, P, R, info, cross, pl.narrow, pl.stride, winstart, winval, pl.max_win, partial, status);
    LAUNCH(K_FINISH, (zl_finish_kernel<256>), dim3((unsigned)(pblocks * B)), dim3(256),
           ts, nullptr, nullptr, P, R, info, (const SegEntry*)(wsp + pl.off_seg), (const void*)cross, pl.narrow, pl.stride,
           partial, pl.max_win, barrier, iters, dmin);
    return EBSP_OK;
}

// Scratch of the entry point that allocates nothing: a file-scope device array that every GPU the
// library runs on holds until the process ends.  In host code the array's name is only a handle
// for hipGetSymbolAddress; its device address is asked for once per device and kept.
static __device__ __align__(256) unsigned char scratch[EBSP_STATIC_SCRATCH_BYTES];

int static_scratch(void** out)
{
    constexpr int KNOWN = 64;
    static std::atomic<void*> base[KNOWN];             // per device: where that GPU's copy of the array lives
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return fail(EBSP_ERR_DEVICE, "no current HIP device");
    if (dev < 0 || dev >= KNOWN) return fail(EBSP_ERR_DEVICE, "device ordinal beyond what the static scratch table holds");
    void* ptr = base[dev].load(std::memory_order_acquire);
    if (!ptr) {
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            snprintf(g_err, sizeof g_err, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
            return EBSP_ERR_DEVICE;
        }
        base[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return EBSP_OK;
}

}  // namespace

extern "C" {

size_t ebsp_zipline_static_scratch_bytes(void) { return (size_t)EBSP_STATIC_SCRATCH_BYTES; }

int ebsp_zipline_batch_static(const int64_t* ts, int64_t B, int32_t P, int32_t R,
                              int64_t* barrier, int32_t* iters, int64_t* wait, int32_t* status, void* stream)
{
    if (!ts && B > 0) return fail(EBSP_ERR_NULL, "ts must not be NULL");
    Plan pl;
    if (!make_plan(B, P, R, pl, SINGLE_MAX, false, true)) return fail(EBSP_ERR_SHAPE, "invalid shape: need B >= 0, P >= 1, R >= 1, P*R < 2^31");
    const size_t need = pl.sweep ? pl.sweep_bytes : (pl.multi ? pl.bytes : 0);
    if (need > (size_t)EBSP_STATIC_SCRATCH_BYTES) {
        snprintf(g_err, sizeof g_err, "this batch needs %zu bytes of scratch, the static scratch holds %zu: "
                 "use fewer instances per call or ebsp_zipline_batch with a workspace", need, (size_t)EBSP_STATIC_SCRATCH_BYTES);
        return EBSP_ERR_WORKSPACE;
    }
    void* ptr = nullptr;
    if (B > 0)
        if (int rc = static_scratch(&ptr)) return rc;
    const int rc = run_batch((const i64*)ts, nullptr, nullptr, B, P, R, (i64*)barrier, iters, (i64*)wait, status,
                             ptr, (size_t)EBSP_STATIC_SCRATCH_BYTES, (hipStream_t)stream);
    if (g_prof.on && rc == EBSP_OK && B > 0 && g_prof.calls < g_prof.max_calls) ++g_prof.calls;
    return rc;
}

size_t ebsp_zipline_workspace_bytes(int64_t B, int32_t P, int32_t R)
{
    Plan pl;
    if (!make_plan(B, P, R, pl, SINGLE_MAX, false, true)) return 0;
    if (pl.sweep) return pl.sweep_bytes;
    return pl.multi ? pl.bytes : 0;
}

size_t ebsp_predict_zipline_workspace_bytes(int64_t B, int32_t P, int32_t R)
{
    Plan pl;
    if (!make_plan(B, P, R, pl)) return 0;
    return pl.multi ? pl.bytes : 0;
}

int ebsp_zipline_batch(const int64_t* ts, int64_t B, int32_t P, int32_t R,
                       int64_t* barrier, int32_t* iters, int64_t* wait,
                       int32_t* status, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!ts && B > 0) return fail(EBSP_ERR_NULL, "ts must not be NULL");
    const int rc = run_batch((const i64*)ts, nullptr, nullptr, B, P, R, (i64*)barrier, iters, (i64*)wait, status,
                             workspace, workspace_bytes, (hipStream_t)stream);
    if (g_prof.on && rc == EBSP_OK && B > 0 && g_prof.calls < g_prof.max_calls) ++g_prof.calls;
    return rc;
}

int ebsp_predict_zipline_batch(const int64_t* last_end, const int64_t* interval, int64_t B, int32_t P, int32_t R,
                               int64_t* barrier, int32_t* iters, int64_t* wait,
                               int32_t* status, void* workspace, size_t workspace_bytes, void* stream)
{
    if ((!last_end || !interval) && B > 0) return fail(EBSP_ERR_NULL, "last_end and interval must not be NULL");
    const int rc = run_batch(nullptr, (const i64*)last_end, (const i64*)interval, B, P, R, (i64*)barrier, iters,
                             (i64*)wait, status, workspace, workspace_bytes, (hipStream_t)stream);
    if (g_prof.on && rc == EBSP_OK && B > 0 && g_prof.calls < g_prof.max_calls) ++g_prof.calls;
    return rc;
}

size_t ebsp_simulate_workspace_bytes(int64_t B, int32_t P, int32_t R)
{
    Plan pl;
    if (!make_plan(B, P, R, pl)) return 0;
    return align_up(pl.multi ? pl.bytes : 0, 256) + align_up((size_t)B * P * sizeof(i64), 256);   // + the workers' current start times
}

int ebsp_simulate_supersteps(const int64_t* last_end0, const int64_t* interval, int64_t sync_cost,
                             int64_t S, int64_t B, int32_t P, int32_t R, int64_t* barrier, int32_t* iters, int64_t* wait, int32_t* status,
                             void* workspace, size_t workspace_bytes, void* stream)
{
    Plan pl;
    if (S < 0 || sync_cost < 0 || !make_plan(B, P, R, pl))
        return fail(EBSP_ERR_SHAPE, "invalid shape: need S >= 0, sync_cost >= 0, B >= 0, P >= 1, R >= 1, P*R < 2^31");
    if (S == 0 || B == 0) return EBSP_OK;
    if (!last_end0 || !interval) return fail(EBSP_ERR_NULL, "last_end0 and interval must not be NULL");
    if (!barrier || !iters || !wait) return fail(EBSP_ERR_NULL, "barrier, iters and wait must not be NULL");
    if (!workspace) return fail(EBSP_ERR_NULL, "the simulation needs a workspace");
    if (((uintptr_t)workspace & 255u) != 0) return fail(EBSP_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    const size_t search_bytes = align_up(pl.multi ? pl.bytes : 0, 256);
    if (workspace_bytes < search_bytes + (size_t)B * P * sizeof(i64))
        return fail(EBSP_ERR_WORKSPACE, "workspace smaller than ebsp_simulate_workspace_bytes()");
    if ((B * (i64)P + 255) / 256 > 0x7fffffffll) return fail(EBSP_ERR_SHAPE, "batch too large for one call");
    hipStream_t st = (hipStream_t)stream;
    i64* start = (i64*)((char*)workspace + search_bytes);
    const i64 per = B * (i64)P;
    for (i64 s = 0; s < S; ++s) {
        const i64* from = s == 0 ? (const i64*)last_end0 : start;
        int* flags = status ? status + s * B : nullptr;
        const int rc = run_batch(nullptr, from, (const i64*)interval + s * per, B, P, R, (i64*)barrier + s * B, iters + s * per,
                                 (i64*)wait + s * B, flags, workspace, search_bytes, st);
        if (rc != EBSP_OK) return rc;
        if (s + 1 < S)       // the workers' start times of the next superstep (after the last one barrier[S-1] says it all)
            LAUNCH(K_ADVANCE, zl_advance_kernel, dim3((unsigned)((per + 255) / 256)), dim3(256),
                   (const i64*)barrier + s * B, (const int*)flags, from, start, (i64)sync_cost, B, P);
        if (g_prof.on && g_prof.calls < g_prof.max_calls) ++g_prof.calls;
    }
    return EBSP_OK;
}

size_t ebsp_gridscan_workspace_bytes(int64_t B, int32_t P, int32_t R, int32_t full)
{
    if (B < 0 || P < 1 || R < 1 || (i64)P * R >= (1ll << 31)) return 0;
    return align_up((size_t)B * (full ? (size_t)P : 1) * sizeof(GridBest), 256);
}

int ebsp_gridscan_batch(const int64_t* ts, int64_t B, int32_t P, int32_t R, int32_t full,
                        int64_t* barrier, int32_t* iters, int64_t* dz, int32_t* status,
                        void* workspace, size_t workspace_bytes, void* stream)
{
    if (B < 0 || P < 1 || R < 1 || (i64)P * R >= (1ll << 31))
        return fail(EBSP_ERR_SHAPE, "invalid shape: need B >= 0, P >= 1, R >= 1, P*R < 2^31");
    if (B == 0) return EBSP_OK;
    if (!ts || !barrier || !iters || !dz) return fail(EBSP_ERR_NULL, "ts, barrier, iters and dz must not be NULL");
    const i64 blocks = B * (full ? (i64)P : 1);
    if (blocks > 0x7fffffffll) return fail(EBSP_ERR_SHAPE, "batch too large for one call");
    if (!workspace) return fail(EBSP_ERR_NULL, "the scans need a workspace");
    if (workspace_bytes < ebsp_gridscan_workspace_bytes(B, P, R, full))
        return fail(EBSP_ERR_WORKSPACE, "workspace smaller than ebsp_gridscan_workspace_bytes()");
    if (((uintptr_t)workspace & 255u) != 0) return fail(EBSP_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    if (int rc = check_device()) return rc;
    hipStream_t st = (hipStream_t)stream;
    GridBest* best = (GridBest*)workspace;
    LAUNCH(K_GRIDSCAN, zl_gridscan_kernel, dim3((unsigned)blocks), dim3(GRID_NT), (const i64*)ts, P, R, full ? 1 : 0, best, status);
    LAUNCH(K_GRIDSCAN_FINISH, zl_gridscan_finish_kernel, dim3((unsigned)B), dim3(GRID_NT), (const i64*)ts, P, R, full ? 1 : 0,
           (const GridBest*)best, (i64*)barrier, iters, (i64*)dz);
    if (g_prof.on && g_prof.calls < g_prof.max_calls) ++g_prof.calls;
    return EBSP_OK;
}

size_t ebsp_zipline_range_workspace_bytes(int64_t B, int32_t P, int32_t R)
{
    Plan pl;
    if (!make_plan(B, P, R, pl, RANGE_SINGLE_MAX, true)) return 0;
    return pl.multi ? pl.bytes : 0;
}

int ebsp_zipline_range_batch(const int64_t* ts, int64_t B, int32_t P, int32_t R,
                             int64_t* barrier, int32_t* iters, int64_t* dmin,
                             int32_t* status, void* workspace, size_t workspace_bytes, void* stream)
{
    const int rc = run_range_batch((const i64*)ts, B, P, R, (i64*)barrier, iters, (i64*)dmin, status,
                                   workspace, workspace_bytes, (hipStream_t)stream);
    if (g_prof.on && rc == EBSP_OK && B > 0 && g_prof.calls < g_prof.max_calls) ++g_prof.calls;
    return rc;
}

int ebsp_zipline_shape_info(int64_t B, int32_t P, int32_t R, int64_t* info)
{
    Plan pl;
    if (!info) return fail(EBSP_ERR_NULL, "info must not be NULL");
    if (!make_plan(B, P, R, pl)) return fail(EBSP_ERR_SHAPE, "invalid shape: need B >= 0, P >= 1, R >= 1, P*R < 2^31");
    info[0] = pl.multi ? 1 : 0;
    info[1] = pl.multi ? pl.cap : 0;
    info[2] = pl.multi ? pl.bins : 0;
    info[3] = pl.multi ? pl.max_win : 0;
    info[4] = pl.multi ? pl.fill : 0;
    Plan stored;
    info[5] = make_plan(B, P, R, stored, SINGLE_MAX, false, true) && stored.sweep ? stored.nslices : 0;
    return EBSP_OK;
}

int ebsp_zipline_tune(int32_t window_cap, int32_t single_max, int32_t window_fill)
{
    if (window_fill < 0 || (window_fill > 0 && window_fill < 512))
        return fail(EBSP_ERR_SHAPE, "window_fill must be 0 or at least 512");
    if (window_cap != 0 && window_cap != 4096 && window_cap != 8192 && window_cap != 16384)
        return fail(EBSP_ERR_SHAPE, "window_cap must be 0, 4096, 8192 or 16384");
    if (single_max < 0 || single_max > SINGLE_MAX)
        return fail(EBSP_ERR_SHAPE, "single_max must be in 0..16384");
    g_tune_window_cap.store(window_cap, std::memory_order_relaxed);
    g_tune_single_max.store(single_max, std::memory_order_relaxed);
    g_tune_window_fill.store(window_fill, std::memory_order_relaxed);
    return EBSP_OK;
}

int ebsp_zipline_tune_sweep(int32_t sweep_min, int32_t slice_keys, int32_t lines)
{
    if (lines < 0 || lines > SWEEP_LINES) return fail(EBSP_ERR_SHAPE, "lines must be in 0..4096");
    if (slice_keys < 0 || (slice_keys > 0 && slice_keys < 256)) return fail(EBSP_ERR_SHAPE, "slice_keys must be 0 or at least 256");
    g_tune_sweep_min.store(sweep_min, std::memory_order_relaxed);
    g_tune_sweep_lines.store(lines, std::memory_order_relaxed);
    g_tune_slice_keys.store(slice_keys, std::memory_order_relaxed);
    return EBSP_OK;
}

int ebsp_zipline_copy_probe(const void* src, void* dst, size_t bytes, void* stream)
{
    if (!src || !dst) return fail(EBSP_ERR_NULL, "src and dst must not be NULL");
    if (bytes == 0 || bytes % 16 != 0 || (((uintptr_t)src | (uintptr_t)dst) & 15u))
        return fail(EBSP_ERR_SHAPE, "copy probe needs a positive multiple of 16 bytes and 16-byte aligned pointers");
    if (int rc = check_device()) return rc;
    hipStream_t st = (hipStream_t)stream;
    const i64 n = (i64)(bytes / 16);
    i64 blocks = (n + 2047) / 2048;                     // pieces of 32 KiB or more
    if (blocks > 256 * 256) blocks = 256 * 256;
    LAUNCH(K_COPY, zl_copy_kernel, dim3((unsigned)blocks), dim3(256), (const uint4*)src, (uint4*)dst, n);
    if (g_prof.on && g_prof.calls < g_prof.max_calls) ++g_prof.calls;
    return EBSP_OK;
}

static_assert(READ_SINK_WORDS == EBSP_READ_SINK_WORDS, "the header's word count is the kernel's");

int ebsp_zipline_read_probe(const void* src, size_t bytes, uint64_t* sink, void* stream)
{
    if (!src || !sink) return fail(EBSP_ERR_NULL, "src and sink must not be NULL");
    if (bytes == 0 || bytes % 16 != 0 || ((uintptr_t)src & 15u) || ((uintptr_t)sink & 7u))
        return fail(EBSP_ERR_SHAPE, "read probe needs a positive multiple of 16 bytes, a 16-byte aligned source and an 8-byte aligned sink of 256 words");
    if (int rc = check_device()) return rc;
    hipStream_t st = (hipStream_t)stream;
    const i64 n = (i64)(bytes / 16);
    i64 blocks = (n + 2047) / 2048;                     // pieces of 32 KiB or more
    if (blocks > 256 * 256) blocks = 256 * 256;
    LAUNCH(K_READ, zl_read_kernel, dim3((unsigned)blocks), dim3(256), (const uint4*)src, n, (u64*)sink);
    if (g_prof.on && g_prof.calls < g_prof.max_calls) ++g_prof.calls;
    return EBSP_OK;
}

int ebsp_zipline_memory_info(int32_t* clock_khz, int32_t* bus_bits)
{
    if (!clock_khz || !bus_bits) return fail(EBSP_ERR_NULL, "clock_khz and bus_bits must not be NULL");
    int dev = 0, clk = 0, bus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return fail(EBSP_ERR_DEVICE, "no current HIP device");
    if (hipDeviceGetAttribute(&clk, hipDeviceAttributeMemoryClockRate, dev) != hipSuccess ||
        hipDeviceGetAttribute(&bus, hipDeviceAttributeMemoryBusWidth, dev) != hipSuccess)
        return fail(EBSP_ERR_DEVICE, "hipDeviceGetAttribute failed");
    *clock_khz = clk;
    *bus_bits = bus;
    return EBSP_OK;
}

int ebsp_zipline_profile_begin(int32_t max_calls)
{
    if (g_prof.on) return fail(EBSP_ERR_SHAPE, "a profile is already open on this thread");
    if (max_calls < 1 || max_calls > 100000) return fail(EBSP_ERR_SHAPE, "max_calls must be in 1..100000");
    const size_t n = (size_t)max_calls * K_COUNT;
    g_prof.ev = new hipEvent_t[2 * n];
    g_prof.used = new bool[n]();
    for (size_t i = 0; i < 2 * n; ++i)
        if (hipEventCreate(&g_prof.ev[i]) != hipSuccess) {
            for (size_t k = 0; k < i; ++k) (void)hipEventDestroy(g_prof.ev[k]);
            delete[] g_prof.ev; delete[] g_prof.used;
            g_prof = Profile();
            return fail(EBSP_ERR_LAUNCH, "hipEventCreate failed");
        }
    g_prof.max_calls = max_calls;
    g_prof.calls = 0;
    g_prof.on = true;
    return EBSP_OK;
}

int ebsp_zipline_profile_end(float* kernel_ms, int32_t* calls)
{
    if (!g_prof.on) return fail(EBSP_ERR_SHAPE, "no profile is open on this thread");
    int rc = EBSP_OK;
    if (hipDeviceSynchronize() != hipSuccess) rc = fail(EBSP_ERR_LAUNCH, "hipDeviceSynchronize failed");
    const size_t n = (size_t)g_prof.max_calls * K_COUNT;
    for (int k = 0; k < K_COUNT && kernel_ms; ++k) kernel_ms[k] = 0.f;
    if (rc == EBSP_OK && kernel_ms)
        for (int c = 0; c < g_prof.calls; ++c)
            for (int k = 0; k < K_COUNT; ++k)
                if (g_prof.used[c * K_COUNT + k]) {
                    float ms = 0.f;
                    const size_t i = ((size_t)c * K_COUNT + k) * 2;
                    if (hipEventElapsedTime(&ms, g_prof.ev[i], g_prof.ev[i + 1]) == hipSuccess) kernel_ms[k] += ms;
                }
    if (calls) *calls = g_prof.calls;
    for (size_t i = 0; i < 2 * n; ++i) (void)hipEventDestroy(g_prof.ev[i]);
    delete[] g_prof.ev;
    delete[] g_prof.used;
    g_prof = Profile();
    return rc;
}

int ebsp_zipline_kernel_count(void) { return K_COUNT; }

const char* ebsp_zipline_kernel_name(int i) { return (i >= 0 && i < K_COUNT) ? kKernelNames[i] : nullptr; }

const char* ebsp_last_error(void) { return g_err; }

}  // extern "C"

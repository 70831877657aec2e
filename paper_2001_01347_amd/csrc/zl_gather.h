// Row segments of a window into (key, delta) records held in registers.
// Part of the ZipLine library (see zipline.hip); device code for gfx950.
#pragma once
#include "zl_bucket.h"

namespace {

// zl_delta for the fast window path: the rows' index ranges are exactly the
// window (no searching), every value of the instance fits 32 bits relative to
// its base, and byte offsets into the instance fit 32 bits.  Two sweeps:
//   1. one thread per row (a round covers 1024 rows): segment lengths, one block
//      scan for the first slots, and a source word for every element of a
//      segment written into that element's slot (index into the instance;
//      FIRST_OF_ROW: the row's very first entry, which has no predecessor;
//      FIRST_OF_SEGMENT: the entry whose predecessor lies before the window).
//      Stored rows: one 32-bit word (29 bits of index, the marks above them);
//      predicted rows: 64 bits (index in the row, marks, row number).
//      The crossing indices of a round are all fetched before any is used.
//   2. one thread per slot: read the source word, load the low words of the
//      element and of its predecessor (GATHER_BATCH elements of a thread in
//      flight together; consecutive slots are consecutive addresses within a
//      segment) and keep the (key, delta) records in registers: item j of
//      thread t is slot j*NT + t.  key = t - (base + a), delta = t - predecessor
//      (the window start for a row's first entry).  W0 = sum_p (a - last value
//      of row p before the window) is collected from the segment-first entries;
//      rows without any entry in the window add their share in sweep 1.
// Returns the number of entries; nothing is loaded if it exceeds `cap`.
constexpr u64 FIRST_OF_ROW = 1ull << 32, FIRST_OF_SEGMENT = 1ull << 33;      // predicted rows
constexpr int PRED_ROW_SHIFT = 34;        // predicted rows: the row number sits above the two flags
constexpr u32 SRC_INDEX = (1u << 29) - 1u, SRC_ROW = 1u << 29, SRC_SEGMENT = 1u << 30, SRC_LAST = 1u << 31;   // stored rows
// rows a thread takes per round of sweep 1: one round covers 1024 rows
template <int NT> constexpr int ROWS_PER_THREAD = NT >= 1024 ? 1 : 1024 / NT;
constexpr int WINDOWS_PER_BLOCK = 2;      // consecutive windows a workgroup handles, one after the other
constexpr u64 HOT_MAX_ENTRIES = 1ull << 29;   // P*R below this: byte offsets into an instance fit 32 bits, indices 29
static_assert(HOT_MAX_ENTRIES - 1 <= SRC_INDEX, "an index must fit its field of the source word");

template <int NT, class CT>
__device__ __forceinline__ void load_ranges(const Rows& rw, int p0, u32 (&lo)[ROWS_PER_THREAD<NT>], u32 (&hi)[ROWS_PER_THREAD<NT>])
{
#pragma unroll
    for (int c = 0; c < ROWS_PER_THREAD<NT>; ++c) {
        const int p = p0 + c * NT + (int)threadIdx.x;
        lo[c] = 0; hi[c] = 0;
        if (p < rw.P) rw.range_as<CT>(p, lo[c], hi[c]);
    }
}

// Sweep 2 for items [g, g + G) of every thread.  Only the low words of the
// timestamps are loaded (rows were checked for order by zl_partition).
// Crossing indices of the thread's rows of the first round at fine bin k (0 for rows beyond P).
template <int NT, class CT>
__device__ __forceinline__ void load_column(const Rows& rw, u32 k, u32 (&out)[ROWS_PER_THREAD<NT>])
{
#pragma unroll
    for (int c = 0; c < ROWS_PER_THREAD<NT>; ++c) {
        const int p = c * NT + (int)threadIdx.x;
        out[c] = 0;
        if (p < rw.P) out[c] = ((const CT*)rw.cr)[(i64)p * rw.stride + k];
    }
}

template <int NT, int ITEMS, int G, bool PRED>
__device__ __forceinline__ void gather_batch(const u64* recs, const char* bytes, const uint2* par, int g, int total,
                                             u32 start, u32 (&key)[ITEMS], u32 (&dl)[ITEMS], u64& w0)
{
    const int tid = threadIdx.x;
    if (g * NT >= total) return;
    u32 cur[G], prv[G];
    if constexpr (PRED) {
        u64 src[G];
#pragma unroll
        for (int j = 0; j < G; ++j) {
            const int q = (g + j) * NT + tid;
            src[j] = q < total ? recs[q] : FIRST_OF_ROW;               // beyond the end: entry 0, harmless
        }
#pragma unroll
        for (int j = 0; j < G; ++j) {
            // the source word holds the row (above the flags) and the index in it
            const uint2 fs = par[(u32)(src[j] >> PRED_ROW_SHIFT)];  // first value of the row, interval
            cur[j] = fs.x + (u32)src[j] * fs.y;
            prv[j] = cur[j] - fs.y;
        }
#pragma unroll
        for (int j = 0; j < G; ++j) {
            const u32 from = (src[j] & FIRST_OF_ROW) ? start : prv[j];
            key[g + j] = cur[j] - start;
            dl[g + j] = cur[j] - from;
            w0 += (src[j] & FIRST_OF_SEGMENT) ? (u64)(start - from) : 0ull;   // below 2^32 like every relative value
        }
    } else {
        const u32* words = (const u32*)recs;
        u32 src[G];
#pragma unroll
        for (int j = 0; j < G; ++j) {
            const int q = (g + j) * NT + tid;
            src[j] = q < total ? words[q] : SRC_ROW;                   // beyond the end: entry 0, harmless
        }
#pragma unroll
        for (int j = 0; j < G; ++j) {
            const u32 at = src[j] & SRC_INDEX;
            const u32 pat = at - (1u - ((src[j] >> 29) & 1u));         // a row's first entry stands in for its predecessor
            cur[j] = *(const u32*)(bytes + (at << 3));
            prv[j] = *(const u32*)(bytes + (pat << 3));
        }
#pragma unroll
        for (int j = 0; j < G; ++j) {
            const u32 from = (src[j] & SRC_ROW) ? start : prv[j];
            key[g + j] = cur[j] - start;
            dl[g + j] = cur[j] - from;
            w0 += (src[j] & SRC_SEGMENT) ? (u64)(start - from) : 0ull;  // below 2^32 like every relative value
        }
    }
}

// Sweep 1 of the window gather (see above): a source word for every entry of the window in
// its slot.  Returns the number of entries (none is written if they exceed `cap`).  For the rows
// without an entry in the window the distances from their last value before it to the window
// start are summed into before_sum and their maximum goes to before_max.  WITH_LAST marks a
// row's very last entry too (stored rows only).
template <int NT, class CT, bool PRED, bool WITH_LAST>
__device__ __forceinline__ int zl_place_rows(const Smem& sm, const Rows& rw, u64 start64, int cap,
                                             const u32 (&lo0)[ROWS_PER_THREAD<NT>], const u32 (&hi0)[ROWS_PER_THREAD<NT>],
                                             u64& before_sum, u32& before_max)
{
    static_assert(!(PRED && WITH_LAST), "the last-of-row mark is for stored rows");
    const u32 start = (u32)start64;                          // low word of the window's first value (absolute)
    const bool wide = rw.wide;                               // the instance's value spread needs more than 32 bits
    const int tid = threadIdx.x;
    u64* recs = sm.recs;
    const char* bytes = (const char*)rw.inst;
    int total = 0;
    constexpr int RPT = ROWS_PER_THREAD<NT>;
    for (int p0 = 0; p0 < rw.P; p0 += RPT * NT) {
        u32 lo[RPT], hi[RPT];
        if (p0 == 0) {                                       // the first round's crossings came with the call
#pragma unroll
            for (int c = 0; c < RPT; ++c) {                  // stale scratch (unsorted rows) cannot lead outside the row
                lo[c] = lo0[c] < (u32)rw.R ? lo0[c] : (u32)rw.R;
                hi[c] = hi0[c] < (u32)rw.R ? hi0[c] : (u32)rw.R;
                hi[c] = hi[c] > lo[c] ? hi[c] : lo[c];
            }
        } else {
            load_ranges<NT, CT>(rw, p0, lo, hi);
        }
        u32 mine = 0;
        u32 before[RPT];                                     // rows with nothing in the window: their last entry before it
#pragma unroll
        for (int c = 0; c < RPT; ++c) {
            const int p = p0 + c * NT + tid;
            mine += hi[c] - lo[c];
            before[c] = start;
            if (p < rw.P && lo[c] == hi[c] && lo[c] > 0) {
                if (PRED) { const uint2 fs = rw.par[p]; before[c] = fs.x + (lo[c] - 1u) * fs.y; }
                else if (!wide) before[c] = *(const u32*)(bytes + (((u32)p * (u32)rw.R + lo[c] - 1u) << 3));
                else       // a worker that finished long ago may stand 2^32 or more before the window: the whole value
                    before_sum += start64 - (u64)*(const i64*)(bytes + (((u32)p * (u32)rw.R + lo[c] - 1u) << 3));
            }
        }
        u32 round;
        u32 slot = (u32)total + block_excl_scan<u32, NT>(mine, (u32*)sm.red, round);
        total += (int)round;
        if (total > cap) return total;                       // the same for every thread: nothing is written
        // The source words of a row's segment, two per trip.  This loop runs as long as the longest
        // segment among a wave's rows, so it is kept to a store and two additions.
#pragma unroll
        for (int c = 0; c < RPT; ++c) {
            const int p = p0 + c * NT + tid;
            const u32 n = hi[c] - lo[c];
            if (p < rw.P && n > 0) {
                if constexpr (PRED) {
                    constexpr u32 SEGMENT_BIT = (u32)(FIRST_OF_SEGMENT >> 32), ROW_BIT = (u32)(FIRST_OF_ROW >> 32);
                    const u32 rest = (u32)p << (PRED_ROW_SHIFT - 32);            // upper word of every entry but the first
                    const u32 first = lo[c];
                    uint2* dst = (uint2*)recs + slot;
                    dst[0] = make_uint2(first, rest | SEGMENT_BIT | (lo[c] == 0 ? ROW_BIT : 0u));
                    u32 i = 1;
                    for (; i + 1 < n; i += 2) {
                        dst[i] = make_uint2(first + i, rest);
                        dst[i + 1] = make_uint2(first + i + 1, rest);
                    }
                    if (i < n) dst[i] = make_uint2(first + i, rest);
                } else {
                    const u32 first = (u32)p * (u32)rw.R + lo[c];
                    const u32 marks = SRC_SEGMENT | (lo[c] == 0 ? SRC_ROW : 0u);
                    u32* dst = (u32*)recs + slot;
                    dst[0] = first | marks;
                    u32 i = 1;
                    for (; i + 1 < n; i += 2) {
                        dst[i] = first + i;
                        dst[i + 1] = first + i + 1;
                    }
                    if (i < n) dst[i] = first + i;
                    if (WITH_LAST && hi[c] == (u32)rw.R)             // the row's very last entry (after the stores above, same thread)
                        dst[n - 1] = (first + n - 1) | (n == 1 ? marks : 0u) | SRC_LAST;
                }
                slot += n;
            }
        }
#pragma unroll
        for (int c = 0; c < RPT; ++c) {                      // below 2^32 in an instance whose value spread is (the others: above)
            const u32 gone = start - before[c];
            before_sum += (u64)gone;
            before_max = gone > before_max ? gone : before_max;   // (only searches of such instances use the maximum)
        }
    }
    __syncthreads();
    return total;
}

template <int NT, int ITEMS, class CT, bool PRED>
__device__ __forceinline__ int zl_delta_rows(const Smem& sm, const Rows& rw, u64 a, int cap,
                                             const u32 (&lo0)[ROWS_PER_THREAD<NT>], const u32 (&hi0)[ROWS_PER_THREAD<NT>],
                                             u32 (&key)[ITEMS], u32 (&dl)[ITEMS], u64& w0)
{
    const u64* recs = sm.recs;
    const char* bytes = (const char*)rw.inst;
    const u32 start = (u32)(rw.base + a);                    // low word of the window's first value
    u32 unused = 0;
    const int total = zl_place_rows<NT, CT, PRED, false>(sm, rw, rw.base + a, cap, lo0, hi0, w0, unused);
    if (total > cap) return total;

    constexpr int G0 = ITEMS < GATHER_BATCH ? ITEMS : GATHER_BATCH;
    gather_batch<NT, ITEMS, G0, PRED>(recs, bytes, rw.par, 0, total, start, key, dl, w0);
    static_assert((ITEMS - G0) % GATHER_TAIL == 0 || ITEMS < GATHER_BATCH, "tail batches must tile the items");
#pragma unroll
    for (int g = G0; g < ITEMS; g += GATHER_TAIL)
        gather_batch<NT, ITEMS, GATHER_TAIL, PRED>(recs, bytes, rw.par, g, total, start, key, dl, w0);
    return total;
}

}  // namespace

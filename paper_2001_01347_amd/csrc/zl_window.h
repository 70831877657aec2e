// Window kernels of the summed-wait search.
// Part of the ZipLine library (see zipline.hip); device code for gfx950.
#pragma once
#include "zl_plan.h"

namespace {

// Where a window sits: instance b, window j, fine bins [k0, k1), values [A, Elast].
struct WinPos {
    i64 b;
    int j;
    bool valid;
    Rows rw;
    u64 A, Elast;
    u32 scale;      // of the linear bucket map over [A, Elast]
    u64 inv52;
};

// Window j of instance b (b < B); `ii` must be info[b].
__device__ __forceinline__ WinPos locate_window(i64 b, int j, const InstInfo& ii, const i64* ts,
                                                const i64* le, const i64* iv, int P, int R,
                                                const void* cross, bool narrow, int stride,
                                                const u32* winstart, const WinVal* winval, int max_win)
{
    WinPos w;
    w.b = b;
    w.j = j;
    w.valid = false;
    if (j >= (int)ii.nwin) return w;
    const u32* ws = winstart + b * (i64)(max_win + 1);
    const WinVal wv = winval[b * (i64)max_win + j];
    w.rw.inst = ts ? ts + b * (i64)P * R : nullptr;
    w.rw.le = le ? le + b * (i64)P : nullptr;
    w.rw.iv = iv ? iv + b * (i64)P : nullptr;
    w.rw.P = P; w.rw.R = R; w.rw.base = (u64)ii.base;
    w.rw.cr = narrow ? (const void*)((const unsigned short*)cross + (b * (i64)P) * stride)
                     : (const void*)((const u32*)cross + (b * (i64)P) * stride);
    w.rw.narrow = narrow;
    w.rw.wide = false;          // (only the fast window search looks at it)
    w.rw.stride = stride;
    w.rw.k0 = ws[j];
    w.rw.k1 = ws[j + 1];
    if (w.rw.k0 > ii.nb) w.rw.k0 = ii.nb;              // stale scratch cannot index outside a row of cross
    if (w.rw.k1 > ii.nb) w.rw.k1 = ii.nb;
    if (w.rw.k1 <= w.rw.k0) w.rw.k1 = w.rw.k0 < ii.nb ? w.rw.k0 + 1 : w.rw.k0;
    w.A = wv.A;                                         // first and last value of the window
    w.Elast = wv.Elast;
    w.scale = wv.scale ? wv.scale : 1u;
    w.inv52 = wv.inv52;
    w.valid = w.Elast >= w.A;
    return w;
}

// LDS of a fast window search.  The record area first holds the source words of the window's
// entries and then the entries that survive the bounds.  Stored rows: 4 bytes per source word, so
// the area is half the size and holds records for half the entries (more survivors than that are
// listed in rounds); with the bucket words after it the LDS of a CU takes three workgroups of 512
// threads (how many run is then a matter of registers: three of the range search, two of the
// summed-wait search, five of its 256-thread form).  EXTRA_WORDS: room behind the source words.
template <int NT, int ITEMS, bool PRED, int EXTRA_WORDS = 0>
struct WinHot {
    using H = HotCfg<NT, ITEMS, false>;                  // windows use the linear bucket map: no coarse table
    static constexpr int LIST = PRED ? 0 : H::CAP / 2;    // records of the compact list (0: one per entry)
    static constexpr size_t REC_BYTES = PRED ? (size_t)H::BSUM_AT * 8 : (size_t)H::CAP * 4 + (size_t)EXTRA_WORDS * 4;
    static constexpr size_t BYTES = REC_BYTES + (size_t)H::NB * 8 + (size_t)H::RED_WORDS * 8 + (size_t)H::NB * 4;
    static_assert(REC_BYTES % 8 == 0, "the bucket words are 8 bytes each");
    __device__ __forceinline__ static Smem carve(unsigned char* smem)
    {
        Smem s;
        s.recs = (u64*)smem;
        s.dhi = nullptr;
        s.red = (u64*)(smem + REC_BYTES) + H::NB;        // bucket words sit between the records and the scratch
        s.cnt = (u32*)(s.red + H::RED_WORDS);
        return s;
    }
};

// The fast search of one window (see zl_window_kernel); lo/hi hold the index
// ranges of the thread's first ROWS_PER_THREAD<NT> rows.
template <int NT, int ITEMS, class CT, bool PRED>
__device__ __forceinline__ void window_search(const Smem& sm, const Rows& rw, const WinVal& wv, const InstInfo& ii, bool hot,
                                              const u32 (&lo)[ROWS_PER_THREAD<NT>], const u32 (&hi)[ROWS_PER_THREAD<NT>],
                                              Partial* __restrict__ out)
{
    using H = HotCfg<NT, ITEMS>;
    {
        u64* bsum = sm.red - H::NB;
        bsum[threadIdx.x] = 0; bsum[threadIdx.x + NT] = 0;
    }
    Partial r;
    r.wait = U64_MAX;
    r.brel = 0;
    if (wv.Elast >= wv.A) {
        // scale 0: zl_plan found the window unfit for 32-bit keys and deltas (a window that wide is among them)
        bool defer = !hot || ((wv.Elast - wv.A) >> 32) != 0 || wv.scale == 0;
        if (!defer) {
            u32 key[ITEMS], dl[ITEMS];
            u64 w0 = 0;
            const int total = zl_delta_rows<NT, ITEMS, CT, PRED>(sm, rw, wv.A, H::CAP, lo, hi, key, dl, w0);
            defer = total > H::CAP;
            if (!defer && total > 0) {
                u32 bkey;
                if (zl_bucket_finish<NT, ITEMS, true, LinearMap, WinHot<NT, ITEMS, PRED>::LIST>(sm, key, StoredDeltas<ITEMS>{dl},
                                                      linear_map((u32)(wv.Elast - wv.A), H::NB, wv.scale ? wv.scale : 1u,
                                                                 wv.inv52),
                                                      SlotsBelow<NT>{total}, wv.A, ii.thr, (u32)rw.P, w0, r.wait, bkey))
                    r.brel = wv.A + bkey;
                else
                    defer = true;
            }
        }
        if (defer) {
            r.wait = U64_MAX;
            r.brel = DEFERRED_WINDOW;
        }
    }
    __syncthreads();                          // everyone is done with LDS before the next window
    if (threadIdx.x == 0) *out = r;
}

// The summed-wait search of one window for window_pairs().
template <int NT, int ITEMS, class CT, bool PRED>
struct SumSearch {
    static constexpr bool PREDICTED = PRED;
    __device__ __forceinline__ static void run(const Smem& sm, const Rows& rw, const WinVal& wv, const InstInfo& ii, bool hot,
                                               const u32 (&lo)[ROWS_PER_THREAD<NT>], const u32 (&hi)[ROWS_PER_THREAD<NT>],
                                               Partial* __restrict__ out)
    {
        window_search<NT, ITEMS, CT, PRED>(sm, rw, wv, ii, hot, lo, hi, out);
    }
};

// One workgroup per WINDOWS_PER_BLOCK consecutive windows of an instance; each
// window's best candidate goes to `partial`.  Handles the normal case (32-bit
// value spread, the window fits in LDS) and marks every other window as deferred
// to the general kernel.  A window's upper crossings are the next window's lower
// ones, and those of the window after are fetched while the current one is
// being searched.  `Search` does one window.
template <int NT, int ITEMS, class CT, class Search>
__device__ __forceinline__ void window_pairs(
    const Smem& sm, const i64* __restrict__ ts, const uint2* __restrict__ rowpar, i64 B, int P, int R,
    const InstInfo* __restrict__ info, const CT* __restrict__ cross, int stride,
    const u32* __restrict__ winstart, const WinVal* __restrict__ winval, int max_win, u32 groups, u32 groups_inv,
    Partial* __restrict__ partial)
{
    constexpr bool PRED = Search::PREDICTED;
    constexpr int RPT = ROWS_PER_THREAD<NT>;
    // Consecutive windows share cache lines at their segment ends: give each
    // XCD (workgroups are dealt round-robin to the 8 XCDs) a contiguous range.
    const u32 per_xcd = gridDim.x / 8;
    const u32 slot = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    // slot = b * groups + group, with groups_inv = floor(2^32 / groups): the estimate is at most one short
    u32 b = __umulhi(slot, groups_inv);
    u32 group = slot - b * groups;
    if (group >= groups) { ++b; group -= groups; }
    if ((i64)b >= B) return;
    const int j0 = (int)group * WINDOWS_PER_BLOCK;
    const u32* ws = winstart + b * (i64)(max_win + 1);       // max_win + 1 entries
    const WinVal* wv = winval + b * (i64)max_win;
    // fine bins where the windows start and end and the windows' values: asked for together
    // with the instance's facts, before anything depends on those (j0 + W <= max_win, so the
    // addresses are valid even where the instance has fewer windows)
    constexpr int W = WINDOWS_PER_BLOCK;
    u32 bins[W + 1];
    WinVal vals[W];
#pragma unroll
    for (int i = 0; i <= W; ++i) bins[i] = ws[j0 + i];
#pragma unroll
    for (int i = 0; i < W; ++i) vals[i] = wv[j0 + i];
    const InstInfo ii = info[b];
    const int jend = j0 + WINDOWS_PER_BLOCK < (int)ii.nwin ? j0 + WINDOWS_PER_BLOCK : (int)ii.nwin;
    if (j0 >= jend) return;
    Partial* out = partial + b * (i64)max_win;
    // The fast search holds keys relative to its window and deltas between neighbours in 32 bits.  That
    // fits every window of an instance whose value spread does; in the others zl_plan has marked the
    // windows it does not fit (WinVal::scale == 0).
    const bool hot = (!(ii.range >> 32) || !PRED) && (u64)P * (u64)R < HOT_MAX_ENTRIES;
    Rows rw;
    rw.inst = PRED ? nullptr : ts + b * (i64)P * R;
    rw.le = nullptr; rw.iv = nullptr;
    rw.par = PRED ? rowpar + b * (i64)P : nullptr;
    rw.P = P; rw.R = R; rw.base = (u64)ii.base;
    rw.cr = (const void*)(cross + (b * (i64)P) * stride);
    rw.narrow = sizeof(CT) == 2;
    rw.wide = (ii.range >> 32) != 0;
    rw.stride = stride;
#pragma unroll
    for (int i = 0; i <= W; ++i)                             // stale scratch cannot index outside a row of cross
        bins[i] = bins[i] < ii.nb ? bins[i] : ii.nb;
    u32 lo[RPT], hi[RPT], next[RPT];
#pragma unroll
    for (int c = 0; c < RPT; ++c) { lo[c] = hi[c] = next[c] = 0; }
    if (hot) {
        load_column<NT, CT>(rw, bins[0], lo);
        load_column<NT, CT>(rw, bins[1], hi);
    }
#pragma unroll
    for (int i = 0; i < W; ++i) {
        if (j0 + i < jend) {
            if (hot && i + 1 < W && j0 + i + 1 < jend) load_column<NT, CT>(rw, bins[i + 1 < W ? i + 2 : W], next);
            rw.k0 = bins[i];
            rw.k1 = bins[i + 1] > bins[i] ? bins[i + 1] : bins[i];
            Search::run(sm, rw, vals[i], ii, hot, lo, hi, out + j0 + i);
#pragma unroll
            for (int c = 0; c < RPT; ++c) { lo[c] = hi[c]; hi[c] = next[c]; }
        }
    }
}

template <int NT, int ITEMS, class CT, bool PRED>
__global__ __launch_bounds__(NT, (!PRED && NT == 256 ? 5 : 4)) void zl_window_kernel(
    const i64* __restrict__ ts, const uint2* __restrict__ rowpar, i64 B, int P, int R,
    const InstInfo* __restrict__ info, const CT* __restrict__ cross, int stride,
    const u32* __restrict__ winstart, const WinVal* __restrict__ winval, int max_win, u32 groups, u32 groups_inv,
    Partial* __restrict__ partial)
{
    using L = WinHot<NT, ITEMS, PRED>;
    __shared__ __align__(16) unsigned char smem[L::BYTES];
    const Smem sm = L::carve(smem);
    window_pairs<NT, ITEMS, CT, SumSearch<NT, ITEMS, CT, PRED>>(sm, ts, rowpar, B, P, R, info, cross, stride, winstart,
                                                               winval, max_win, groups, groups_inv, partial);
}

// The windows zl_window_kernel deferred: the general window search.  A small
// fixed grid; every workgroup looks through its share of the window results for
// deferred marks and handles the marked windows one after the other.
template <int NT, int ITEMS>
__global__ __launch_bounds__(NT) void zl_window_general_kernel(
    const i64* __restrict__ ts, const i64* __restrict__ le, const i64* __restrict__ iv, i64 B, int P, int R,
    const InstInfo* __restrict__ info, const void* __restrict__ cross, bool narrow, int stride,
    const u32* __restrict__ winstart, const WinVal* __restrict__ winval, int max_win,
    Partial* __restrict__ partial, int* __restrict__ status)
{
    using C = WinCfg<NT, ITEMS>;
    __shared__ __align__(16) unsigned char smem[C::BYTES];
    const Smem sm = carve<NT, ITEMS>(smem);
    const u32 total = (u32)(B * (i64)max_win);
    const u32 share = (total + gridDim.x - 1) / gridDim.x;
    const u32 first = blockIdx.x * share;
    const u32 end = first + share < total ? first + share : total;

    for (u32 base = first; base < end; base += NT) {
        const u32 idx = base + threadIdx.x;
        bool mine = false;
        if (idx < end) {
            const u32 b = idx / (u32)max_win, j = idx % (u32)max_win;
            if (j < info[b].nwin) mine = partial[idx].wait == U64_MAX && partial[idx].brel == DEFERRED_WINDOW;
        }
        for (;;) {
            const u32 pick = block_reduce<u32, NT>(mine ? idx : 0xffffffffu, (u32*)sm.red, OpMin());
            if (pick == 0xffffffffu) break;
            if (pick == idx) mine = false;
            const i64 pb = pick / (u32)max_win;
            const InstInfo ii = info[pb];
            const WinPos w = locate_window(pb, (int)(pick % (u32)max_win), ii, ts, le, iv, P, R, cross, narrow, stride,
                                           winstart, winval, max_win);
            u64 bw = U64_MAX, bb = 0;
            int bad = 0;
            if (w.valid) {
                // the 64-bit-delta form serves every deferred window, narrow ones included
                zl_window<NT, ITEMS, true>(sm, w.rw, ii.thr, w.A, w.Elast, bw, bb, bad);
            }
            bad = __syncthreads_or(bad);
            if (threadIdx.x == 0) {
                Partial r;
                r.wait = bw;
                r.brel = bb;
                partial[pick] = r;
                if (bad && status) atomicOr(status + w.b, (int)EBSP_STATUS_UNSORTED);
            }
        }
    }
}

}  // namespace

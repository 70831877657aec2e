// The general search of one value interval, walked in pieces that fit a workgroup.
// Part of the ZipLine library (see zipline.hip); device code for gfx950.
#pragma once
#include "zl_gather.h"

namespace {

// Number of entries of the rows inside [a, el].
template <int NT>
__device__ __forceinline__ u32 count_interval(const Smem& sm, const Rows& rw, u64 a, u64 el, bool lx)
{
    u32 c = 0;
    for (int p = threadIdx.x; p < rw.P; p += NT) {
        u32 lo, hi;
        sub_range(rw, p, a, el, lx, false, lo, hi);
        c += hi - lo;
    }
    return block_reduce<u32, NT>(c, (u32*)sm.red, OpAdd());
}

// Search one value interval [A, Elast] of the rows in `rw`: the general form of
// zl_delta -> zl_sort -> zl_scan -> zl_argmin.  Normally the interval is at
// most 2^32 wide (any width with KEY64: 64-bit keys, their upper halves in a third
// plane) and holds at most `cap` entries and is handled in one go.
// Otherwise it is walked in pieces that do fit, cut by bisection on the value;
// a single value that alone occurs more than `cap` times is one candidate and
// is evaluated directly from the rows.  (bw, bb) is updated with the first
// minimum found: smaller wait, then smaller barrier (relative to base).
template <int NT, int ITEMS, bool WIDE, bool KEY64 = false>
__device__ __forceinline__ void zl_window(const Smem& sm, const Rows& rw, u64 thr, u64 A, u64 Elast,
                                          u64& bw, u64& bb, int& bad)
{
    using C = WinCfg<NT, ITEMS>;
    constexpr int CAPW = WIDE ? C::CAP_WIDE : C::CAP;
    u64 a = A;
    bool lx = true;
    for (;;) {
        u64 el = Elast;
        bool rx = true;
        if (!KEY64 && el - a > 0xffffffffull) { el = a + 0xffffffffull; rx = false; }
        u64 w0 = 0;
        int total = zl_delta<NT, WIDE, true, KEY64>(sm, rw, a, el, lx, rx, CAPW, w0, bad);
        bool single = false;
        if (total > CAPW) {
            if (count_interval<NT>(sm, rw, a, a, lx) > (u32)CAPW) {
                single = true;                     // the value `a` alone overflows a window
                el = a;
            } else {
                u64 l = a, h = el;                 // count(a, l) <= CAPW < count(a, h)
                while (h - l > 1) {
                    const u64 m = l + ((h - l) >> 1);
                    if (count_interval<NT>(sm, rw, a, m, lx) <= (u32)CAPW) l = m; else h = m;
                }
                el = l;
                w0 = 0;
                total = zl_delta<NT, WIDE, true, KEY64>(sm, rw, a, el, lx, false, CAPW, w0, bad);
            }
            rx = false;
        }
        if (single) {
            // candidate c = a: every row stops at its last entry <= a
            u64 s = 0;
            int missing = 0;
            for (int p = threadIdx.x; p < rw.P; p += NT) {
                u32 lo, hi;
                sub_range(rw, p, a, a, lx, false, lo, hi);
                if (hi > 0) s += a - rw.rel(p, hi - 1); else missing = 1;
            }
            const u64 w = block_reduce<u64, NT>(s, sm.red, OpAdd());
            missing = __syncthreads_or(missing);
            if (!missing && a >= thr && (w < bw || (w == bw && a < bb))) { bw = w; bb = a; }
        } else if (total > 0) {
            const int items = (total + NT - 1) / NT;
            fill_sentinels<NT>(sm.recs, total, items);
            if (KEY64) fill_sentinels_hi<NT>(sm.ext, total, items);
            const u64 W0 = block_reduce<u64, NT>(w0, sm.red, OpAdd());   // also orders the record writes
            zl_sort<NT, ITEMS, WIDE, KEY64, KEY64>(sm, items, bit_length(el - a));
            u64 w, key;
            zl_scan_argmin<NT, WIDE, KEY64>(sm, items, total, a, thr, (u64)rw.P, W0, w, key);
            if (w != U64_MAX && (w < bw || (w == bw && a + key < bb))) { bw = w; bb = a + key; }
        }
        if (rx) break;
        // continue at the smallest entry above el, if any
        u64 nxt = U64_MAX;
        int have = 0;
        if (el != U64_MAX) {
            for (int p = threadIdx.x; p < rw.P; p += NT) {
                u32 lo, hi;
                rw.range(p, lo, hi);
                const u32 i = row_lower_bound(rw, p, lo, hi, el + 1);
                if (i < hi) { const u64 v = rw.rel(p, i); nxt = v < nxt ? v : nxt; have = 1; }
            }
        }
        nxt = block_reduce<u64, NT>(nxt, sm.red, OpMin());
        have = __syncthreads_or(have);
        if (!have || nxt > Elast || nxt <= el) break;
        a = nxt;
        lx = false;
    }
}

}  // namespace

// The integer maps of the search: the fine-bin grid of an instance, the value buckets of a window (LinearMap) and of
// a whole instance (TableMap), and the bounds on a bucket's keys that the pruning relies on.
// Plain integer arithmetic with no device intrinsics, so that a host program can check it value by value: the
// includer defines ZL_FN (the function qualifiers) first.
// Part of the ZipLine library (see zipline.hip).
#pragma once
#include <stdint.h>

typedef unsigned long long u64;
typedef unsigned int u32;
typedef unsigned short u16;
typedef long long i64;

namespace {

// Per-instance facts shared by the kernels of the multi-window path.
struct InstInfo {
    i64 base;    // min_p t[p][0]; all other values are relative to it
    u64 range;   // max_p t[p][R-1] - base
    u64 thr;     // max_p t[p][0] - base: earliest admissible barrier
    u32 segshift; // segment of the fine-bin map that (v >> wshift) falls in: (v >> wshift) >> segshift
    u32 wshift;  // 0 unless the range needs more than 32 bits
    u32 nb;      // number of fine bins, bin(range) + 1
    u32 nwin;    // number of windows (set by zl_plan)
    u32 flags;   // EBSP_STATUS_* bits found so far
    u32 wide_steps; // how often a row steps by 2^32 or more from one entry to the next (counted by zl_partition)
};
constexpr u32 WIDE_MARKS = 15;   // of those steps, as many are remembered per instance by the fine bin they end in

ZL_FN int bit_length(u64 x) { return x ? 64 - __builtin_clzll(x) : 0; }

// Fine-bin grid of an instance: a monotone map of relative values onto [0, nb).
// x = v >> wshift runs over SEGS segments of 2^segshift values each; within segment s
// the bin is (G[s] + offset * slope[s]) >> 32 with G[s + 1] = G[s] + 2^segshift *
// slope[s] (32.32 fixed point), so the map is continuous and never decreases.
// zl_bounds sets the slopes from an estimate of how many entries each segment holds
// (rows taken as evenly spaced between their first and last value), so that bins
// hold about the same number of entries wherever the rows are dense or sparse.
constexpr int SEGS = 64;
struct SegEntry {        // one segment of an instance's map
    u64 G;
    u32 slope;
    u32 pad_;
};
ZL_FN u32 fine_bin(u64 rel, const InstInfo& ii, const SegEntry* tab)
{
    if (rel > ii.range) rel = ii.range;              // only reachable for unsorted rows
    const u32 x = (u32)(rel >> ii.wshift);
    const u32 s = x >> ii.segshift;
    const SegEntry e = tab[s];
    const u32 k = (u32)((e.G + (u64)(x - (s << ii.segshift)) * e.slope) >> 32);
    return k < ii.nb ? k : ii.nb - 1;
}
// Smallest relative value that falls in bin k or later (k < nb).
ZL_FN u64 fine_bin_start(u32 k, const InstInfo& ii, const SegEntry* tab)
{
    const u64 wmax = (1ull << ii.segshift) - 1;
    const u64 want = (u64)k << 32;
    int lo = 0, hi = SEGS - 1;                       // first segment whose last value reaches bin k
    while (lo < hi) {
        const int m = (lo + hi) >> 1;
        const SegEntry e = tab[m];
        if (((e.G + wmax * e.slope) >> 32) >= k) hi = m; else lo = m + 1;
    }
    const SegEntry e = tab[lo];
    u64 off = 0;
    if (want > e.G && e.slope) off = (want - e.G + e.slope - 1) / e.slope;
    return (((u64)lo << ii.segshift) + off) << ii.wshift;
}


// Slope (bins per value of x, 32.32 fixed point, rounded down) of a segment that is to get the share
// (est + even) / total2 of the bins - 1 bins of the grid over its `len` values in use.
ZL_FN u32 seg_slope_of(u64 est, u64 even, u64 total2, int bins, u64 len)
{
    const double share = (double)(est + even) / (double)total2 * (double)(bins - 1);
    const double sl = share * 4294967296.0 / (double)len;
    return sl < 4294967295.0 ? (u32)sl : 0xffffffffu;
}

// Division of many 32-bit numbers by one divisor d >= 2: with m = floor((2^32 - 1) / d) + 1 (one division, once)
// m * d - 2^32 lies in [0, d), so for every n below 2^32 the upper word of n * m is floor(n / d) or one more,
// and one comparison settles it.  (d = 1 has no such m in 32 bits: row_reciprocal gives 0 and the caller divides.)
ZL_FN u32 row_reciprocal(u64 d) { return (d >> 32) == 0 && (u32)d > 1u ? 0xffffffffu / (u32)d + 1u : 0u; }
ZL_FN u32 div_by_reciprocal(u32 n, u32 d, u32 m)
{
    const u32 q = (u32)(((u64)n * (u64)m) >> 32);
    return q - ((u64)q * (u64)d > (u64)n ? 1u : 0u);
}

// Monotone maps of keys onto value buckets [0, NB).
// LinearMap: bucket = (key * scale) >> 32, equal slices of [0, span]; right when the
// keys are spread evenly, as inside a window of the multi-window path.
// (Keys beyond the span only occur in unsorted rows; the clamps keep those in bounds.)
struct LinearMap {
    u32 scale, top;
    u32 span;      // largest key of sorted rows
    u64 inv52;     // floor(2^52 / scale)
    static constexpr bool HAS_BOUNDS = true;
    ZL_FN u32 operator()(u32 key) const
    {
        const u32 b = (u32)(((u64)key * scale) >> 32);
        return b < top ? b : top;
    }
    // lo <= every key of bucket b <= hi (for keys within [0, span]).  A key k of bucket
    // b < top has b * 2^32 <= k * scale < (b + 1) * 2^32; inv52 is at most one short of
    // 2^52 / scale, which costs less than 2 after the shift (b + 1 <= 2^11).
    ZL_FN void bounds(u32 b, u32& lo, u32& hi) const
    {
        const u64 l = ((u64)b * inv52) >> 20;
        const u64 h = (((u64)(b + 1) * inv52) >> 20) + 2;
        hi = (b >= top || h > span) ? span : (u32)h;
        lo = l > hi ? hi : (u32)l;
    }
    // The same for buckets b and b + 1 with one product: floor((b + 1) * x) >= floor(b * x) +
    // floor(x), and a bucket is less than floor(x) + 2 wide (x = inv52 / 2^20).
    ZL_FN void bounds_pair(u32 b, u32& lo0, u32& hi0, u32& lo1, u32& hi1) const
    {
        const u64 step = inv52 >> 20;
        const u64 l0 = ((u64)b * inv52) >> 20, l1 = l0 + step;
        const u64 h0 = l0 + step + 4, h1 = l1 + step + 4;
        hi0 = h0 > span ? span : (u32)h0;
        hi1 = (b + 1 >= top || h1 > span) ? span : (u32)h1;
        lo0 = l0 > hi0 ? hi0 : (u32)l0;
        lo1 = l1 > hi1 ? hi1 : (u32)l1;
    }
};
ZL_FN u32 linear_scale(u64 span, u32 nb)
{
    const u64 q = ((u64)nb << 32) / (span + 1);
    return q >= 0xffffffffull ? 0xffffffffu : (q ? (u32)q : 1u);
}
ZL_FN LinearMap linear_map(u32 span, u32 nb, u32 scale, u64 inv52)
{
    LinearMap m;
    m.scale = scale;
    m.top = nb - 1;
    m.span = span;
    m.inv52 = inv52;
    return m;
}
// TableMap: piecewise linear through up to 256 coarse bins of width 2^cshift, each
// given a share of the buckets in proportion to its key count, so that buckets
// hold about the same number of keys even where the density of keys varies (a
// whole instance: many workers early in the value range, few stragglers late).
// tab[c] = first bucket of coarse bin c | (buckets of bin c scaled by 2^(32-cshift)) << 32.
template <bool BOUNDS>       // whether the caller wants to drop buckets by their bounds
struct TableMap {
    const u64* tab;     // 256 entries, followed by 256 of: buckets of the bin << 52 | floor(2^52 / multiplier)
    u32 cshift, cmask;
    u32 span;           // largest key of sorted rows
    static constexpr bool HAS_BOUNDS = BOUNDS;
    ZL_FN u32 coarse(u32 key) const { const u32 c = key >> cshift; return c < 255u ? c : 255u; }
    ZL_FN u32 operator()(u32 key) const
    {
        const u64 e = tab[coarse(key)];
        return (u32)e + (u32)(((u64)(key & cmask) * (e >> 32)) >> 32);
    }
    // lo <= every key of bucket b <= hi.  The bins that reach bucket b are consecutive:
    // the lower bound comes from the first of them, the upper bound from the last; inside
    // a bin the bucket is linear in the key's low bits, as for LinearMap.
    ZL_FN void bounds(u32 b, u32& lo, u32& hi) const
    {
        const u64* inv = tab + 256;
        int l = 0, h = 255;
        while (l < h) {                                    // last bin whose first bucket is <= b
            const int m = (l + h + 1) >> 1;
            if ((u32)tab[m] <= b) l = m; else h = m - 1;
        }
        const int chi = l;
        l = 0; h = chi;
        while (l < h) {                                    // first bin whose last bucket is >= b
            const int m = (l + h) >> 1;
            if ((u32)tab[m] + (u32)(inv[m] >> 52) > b) h = m; else l = m + 1;
        }
        const int clo = l;
        const u64 ilo = inv[clo] & ((1ull << 52) - 1), ihi = inv[chi] & ((1ull << 52) - 1);
        const u32 first_lo = (u32)tab[clo], first_hi = (u32)tab[chi];
        const u32 rlo = b >= first_lo ? b - first_lo : 0u, rhi = b >= first_hi ? b - first_hi : 0u;   // below 2^11
        u64 xl = ((u64)rlo * ilo) >> 20, xh = (((u64)(rhi + 1) * ihi) >> 20) + 2;
        xl = xl > cmask ? cmask : xl;
        xh = xh > cmask ? cmask : xh;
        const u64 kh = ((u64)chi << cshift) + xh, kl = ((u64)clo << cshift) + xl;
        hi = kh > span ? span : (u32)kh;
        lo = kl > hi ? hi : (u32)kl;
    }
    ZL_FN void bounds_pair(u32 b, u32& lo0, u32& hi0, u32& lo1, u32& hi1) const
    {
        bounds(b, lo0, hi0);
        bounds(b + 1, lo1, hi1);
    }
};

// One coarse bin of a TableMap over NB buckets: the bin holds `c` of the n keys and `below` keys lie in the bins
// before it.  tab_word goes to tab[bin], inv_word to tab[256 + bin].
ZL_FN void table_entry(u32 below, u32 c, u32 n, u32 NB, u32 cshift, u64& tab_word, u64& inv_word)
{
    const u32 first = (u32)((u64)below * NB / n);
    u32 last = (u32)((u64)(below + c) * NB / n);            // first bucket of the next coarse bin
    if (last > NB - 1) last = NB - 1;
    u32 nbk = last >= first ? last - first + 1 : 1;           // buckets this bin spreads over
    if (cshift < 32 && nbk > (1u << cshift)) nbk = 1u << cshift;
    const u64 mult = cshift ? ((u64)nbk << (32 - cshift)) - 1 : 0ull;
    tab_word = (u64)(first < NB ? first : NB - 1) | (mult << 32);
    inv_word = ((u64)nbk << 52) | (mult ? (1ull << 52) / mult : 0ull);
}

}  // namespace

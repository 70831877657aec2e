// Rows of one instance (stored or predicted) with their index ranges; iteration counts by binary search.
// Part of the ZipLine library (see zipline.hip); device code for gfx950.
#pragma once
#include "zl_common.h"

namespace {

// Rows of one instance and, per row, the index range under consideration:
// the whole row, or [cross[p][k0], cross[p][k1]) from zl_partition.
struct Rows {
    const i64* inst;    // the instance's stored matrix, or nullptr for predicted rows:
    const i64* le;      // t[p][i] = le[p] + (i + 1) * iv[p]   (Section III: iterations of a worker
    const i64* iv;      // take similar time; its next R end timestamps from the last one and the interval)
    const uint2* par;   // predicted rows on the fast window path: low words of (first value, interval) per row
    int P, R;
    u64 base;
    const void* cr;     // crossing indices of this instance (u16 if narrow, else u32), or nullptr for whole rows
    bool narrow;
    bool wide;          // fast window path: the instance's value spread is 2^32 or more
    int stride;
    u32 k0, k1;

    __device__ __forceinline__ void range(int p, u32& lo, u32& hi) const
    {
        if (!cr) { lo = 0; hi = (u32)R; return; }
        if (narrow) {
            const unsigned short* c = (const unsigned short*)cr + (i64)p * stride;
            lo = c[k0]; hi = c[k1];
        } else {
            const u32* c = (const u32*)cr + (i64)p * stride;
            lo = c[k0]; hi = c[k1];
        }
        lo = lo < (u32)R ? lo : (u32)R;               // stale scratch (unsorted rows) cannot
        hi = hi < (u32)R ? hi : (u32)R;               // lead outside the row
        hi = hi > lo ? hi : lo;
    }
    // the same when the caller knows the index type at compile time
    template <class CT>
    __device__ __forceinline__ void range_as(int p, u32& lo, u32& hi) const
    {
        const CT* c = (const CT*)cr + (i64)p * stride;
        lo = c[k0]; hi = c[k1];
        lo = lo < (u32)R ? lo : (u32)R;
        hi = hi < (u32)R ? hi : (u32)R;
        hi = hi > lo ? hi : lo;
    }
    __device__ __forceinline__ i64 value(int p, u32 i) const
    {
        return inst ? inst[(size_t)p * R + i] : (i64)((u64)le[p] + (u64)(i + 1) * (u64)iv[p]);
    }
    __device__ __forceinline__ u64 rel(int p, u32 i) const { return (u64)value(p, i) - base; }
};

// First index in [lo, hi) of row p whose relative value is >= v (hi if none).
__device__ __forceinline__ u32 row_lower_bound(const Rows& rw, int p, u32 lo, u32 hi, u64 v)
{
    while (lo < hi) {
        const u32 m = (lo + hi) >> 1;
        if (rw.rel(p, m) < v) lo = m + 1; else hi = m;
    }
    return lo;
}

// Index range of row p inside the value interval [a, el] (both inclusive).
// lx / rx: the interval starts / ends exactly where the row ranges do.
__device__ __forceinline__ void sub_range(const Rows& rw, int p, u64 a, u64 el, bool lx, bool rx,
                                          u32& lo, u32& hi)
{
    rw.range(p, lo, hi);
    if (!lx) lo = row_lower_bound(rw, p, lo, hi, a);
    if (!rx && el != U64_MAX) hi = row_lower_bound(rw, p, lo, hi, el + 1);
}

// ---------------------------------------------------------------------------
// zl_iters: number of entries of a sorted row that are <= v.
__device__ __forceinline__ int zl_iters(const i64* __restrict__ row, int R, i64 v)
{
    u32 lo = 0, hi = (u32)R;               // unsigned: lo + hi may pass 2^31
    while (lo < hi) {
        const u32 m = (lo + hi) >> 1;
        if (row[m] <= v) lo = m + 1; else hi = m;
    }
    return (int)lo;
}

// The same for row p of stored (inst != nullptr) or predicted rows.
__device__ __forceinline__ int zl_iters_of(const i64* inst, const i64* le, const i64* iv, int p, int R, i64 v)
{
    if (inst) return zl_iters(inst + (size_t)p * R, R, v);
    const i64 l = le[p], s = iv[p];
    u32 lo = 0, hi = (u32)R;
    while (lo < hi) {
        const u32 m = (lo + hi) >> 1;
        if ((i64)((u64)l + (u64)(m + 1) * (u64)s) <= v) lo = m + 1; else hi = m;
    }
    return (int)lo;
}

}  // namespace

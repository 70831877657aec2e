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
//     contiguous segment of every row.  A window that fits in LDS is sorted,
//     scanned and reduced by one workgroup, and the value of the prefix at the
//     window start is known from the row elements just before the segments,
//     so windows need no carry from one another;
//   * small instances (P*R <= 16384) are one window: one workgroup each, no
//     scratch memory, one kernel.
//
// Device steps, named as in the design notes:
//   zl_delta   load a window's row segments, form (key, delta) records
//   zl_sort    LSD radix sort of the records in LDS (wave-ballot ranking)
//   zl_scan    prefix sum of the deltas in sorted order (wave shuffles)
//   zl_argmin  wait(c) at the last element of every run of equal keys,
//              masked to c >= max_p t[p][0]; first minimum wins
//   zl_iters   per-worker iteration counts by binary search
// plus, for instances larger than one window: zl_bounds (instance range),
// zl_partition (row/bin crossing indices), zl_bincount + zl_plan (windows).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>
#include <limits>

#include "ebsp_zipline.h"

typedef unsigned long long u64;
typedef unsigned int u32;
typedef unsigned short u16;
typedef long long i64;

namespace {

constexpr int WAVE = 64;
constexpr u64 U64_MAX = ~0ull;
constexpr i64 DEFERRED = INT64_MIN;            // wait[b] of an instance left to the general kernel
constexpr u64 DEFERRED_WINDOW = ~0ull - 1;      // Partial::brel of a window left to the general kernel

// ---------------------------------------------------------------------------
// Tunables of the multi-window path.
constexpr int LARGE_NT = 1024;               // threads of a general-path workgroup
constexpr int LARGE_ITEMS = 16;              // records per thread
constexpr int SINGLE_MAX = LARGE_NT * LARGE_ITEMS;  // largest P*R one workgroup takes whole
constexpr int GENERAL_GRID = 256;            // workgroups of a general-path kernel (one per CU)
// A window workgroup holds up to `cap` records (4096, 8192 or 16384).  Windows are
// cut every cap/2 keys out of fine bins that hold at most cap/8 keys on average.

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
    u32 pad_;
};

struct Partial {  // best candidate of one window
    u64 wait;     // U64_MAX: the window has no admissible candidate
    u64 brel;     // barrier relative to base
};

// ---------------------------------------------------------------------------
// Wave and block primitives (wave64).

// Cross-lane moves inside the vector ALU (data-parallel primitives): no trip
// through the LDS pipeline.  dpp_take<CTRL, ROWS>(fill, v) gives every lane the
// value of the lane that CTRL selects; lanes in rows outside the ROWS mask and
// lanes whose source does not exist get `fill`.
template <int CTRL, int ROWS>
__device__ __forceinline__ u32 dpp_word(u32 fill, u32 v)
{
    return (u32)__builtin_amdgcn_update_dpp((int)fill, (int)v, CTRL, ROWS, 0xf, false);
}
template <int CTRL, int ROWS, class T>
__device__ __forceinline__ T dpp_take(T fill, T v)
{
    static_assert(sizeof(T) == 4 || sizeof(T) == 8, "one or two words");
    if constexpr (sizeof(T) == 4) {
        return (T)dpp_word<CTRL, ROWS>((u32)fill, (u32)v);
    } else {
        const u64 f = (u64)fill, x = (u64)v;
        return (T)((u64)dpp_word<CTRL, ROWS>((u32)f, (u32)x) |
                   ((u64)dpp_word<CTRL, ROWS>((u32)(f >> 32), (u32)(x >> 32)) << 32));
    }
}
constexpr int DPP_ROW_SHR1 = 0x111, DPP_ROW_SHR2 = 0x112, DPP_ROW_SHR4 = 0x114, DPP_ROW_SHR8 = 0x118,
              DPP_ROW_BCAST15 = 0x142, DPP_ROW_BCAST31 = 0x143,
              DPP_WAVE_SHR1 = 0x138;      // every lane takes the value of the lane before it (across rows)

struct OpMin {
    template <class T> __device__ T operator()(T a, T b) const { return a < b ? a : b; }
    template <class T> static constexpr T identity() { return std::numeric_limits<T>::max(); }
};
struct OpMax {
    template <class T> __device__ T operator()(T a, T b) const { return a > b ? a : b; }
    template <class T> static constexpr T identity() { return std::numeric_limits<T>::lowest(); }
};
struct OpAdd {
    template <class T> __device__ T operator()(T a, T b) const { return a + b; }
    template <class T> static constexpr T identity() { return T(0); }
};

// Inclusive scan over the 64 lanes of a wave: four steps inside each row of 16
// lanes, then the row totals are passed on (last lane of row 0 and 2 to rows 1
// and 3, last lane of row 1 to rows 2 and 3).  Lane 63 ends with the reduction.
template <class T, class Op>
__device__ __forceinline__ T wave_scan(T v, Op op)
{
    constexpr T id = Op::template identity<T>();
    v = op(v, dpp_take<DPP_ROW_SHR1, 0xf>(id, v));
    v = op(v, dpp_take<DPP_ROW_SHR2, 0xf>(id, v));
    v = op(v, dpp_take<DPP_ROW_SHR4, 0xf>(id, v));
    v = op(v, dpp_take<DPP_ROW_SHR8, 0xf>(id, v));
    v = op(v, dpp_take<DPP_ROW_BCAST15, 0xa>(id, v));
    v = op(v, dpp_take<DPP_ROW_BCAST31, 0xc>(id, v));
    return v;
}
template <class T>
__device__ __forceinline__ T wave_incl_scan(T v) { return wave_scan(v, OpAdd()); }

// First minimum of (w, k) pairs over a wave (smaller w, then smaller k); lane 63 ends with it.
template <class K>
__device__ __forceinline__ void wave_argmin(u64& w, K& k)
{
    auto step = [&](u64 ow, K ok) { if (ow < w || (ow == w && ok < k)) { w = ow; k = ok; } };
    constexpr K kmax = std::numeric_limits<K>::max();
    step(dpp_take<DPP_ROW_SHR1, 0xf>(U64_MAX, w), dpp_take<DPP_ROW_SHR1, 0xf>(kmax, k));
    step(dpp_take<DPP_ROW_SHR2, 0xf>(U64_MAX, w), dpp_take<DPP_ROW_SHR2, 0xf>(kmax, k));
    step(dpp_take<DPP_ROW_SHR4, 0xf>(U64_MAX, w), dpp_take<DPP_ROW_SHR4, 0xf>(kmax, k));
    step(dpp_take<DPP_ROW_SHR8, 0xf>(U64_MAX, w), dpp_take<DPP_ROW_SHR8, 0xf>(kmax, k));
    step(dpp_take<DPP_ROW_BCAST15, 0xa>(U64_MAX, w), dpp_take<DPP_ROW_BCAST15, 0xa>(kmax, k));
    step(dpp_take<DPP_ROW_BCAST31, 0xc>(U64_MAX, w), dpp_take<DPP_ROW_BCAST31, 0xc>(kmax, k));
}

// Exclusive block scan; `total` receives the block sum.  `red` holds NT/64 T's.
template <class T, int NT>
__device__ __forceinline__ T block_excl_scan(T v, T* red, T& total)
{
    constexpr int NW = NT / WAVE;
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x >> 6;
    T inc = wave_incl_scan(v);
    if (lane == WAVE - 1) red[wave] = inc;
    __syncthreads();
    T base = 0, sum = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        T x = red[w];
        if (w < wave) base += x;
        sum += x;
    }
    __syncthreads();
    total = sum;
    return base + inc - v;
}

template <class T, int NT, class Op>
__device__ __forceinline__ T block_reduce(T v, T* red, Op op)
{
    constexpr int NW = NT / WAVE;
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x >> 6;
    v = wave_scan(v, op);
    if (lane == WAVE - 1) red[wave] = v;
    __syncthreads();
    T r = red[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) r = op(r, red[w]);
    asm volatile("" : "+v"(r));      // finish the reduction here, not wherever the result is first used
    __syncthreads();
    return r;
}

// min of a, max of b, max of c over the block in one exchange.  `red` holds 3*NT/64 words.
template <int NT>
__device__ __forceinline__ void block_bounds(i64 a, i64 b, i64 c, i64* red, i64& amin, i64& bmax, i64& cmax)
{
    constexpr int NW = NT / WAVE;
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x >> 6;
    a = wave_scan(a, OpMin());
    b = wave_scan(b, OpMax());
    c = wave_scan(c, OpMax());
    if (lane == WAVE - 1) { red[wave] = a; red[NW + wave] = b; red[2 * NW + wave] = c; }
    __syncthreads();
    a = red[0]; b = red[NW]; c = red[2 * NW];
#pragma unroll
    for (int w = 1; w < NW; ++w) {
        const i64 oa = red[w], ob = red[NW + w], oc = red[2 * NW + w];
        a = oa < a ? oa : a;
        b = ob > b ? ob : b;
        c = oc > c ? oc : c;
    }
    __syncthreads();
    amin = a; bmax = b; cmax = c;
}

__device__ __forceinline__ int bit_length(u64 x) { return x ? 64 - __clzll((long long)x) : 0; }

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
__device__ __forceinline__ u32 fine_bin(u64 rel, const InstInfo& ii, const SegEntry* tab)
{
    if (rel > ii.range) rel = ii.range;              // only reachable for unsorted rows
    const u32 x = (u32)(rel >> ii.wshift);
    const u32 s = x >> ii.segshift;
    const SegEntry e = tab[s];
    const u32 k = (u32)((e.G + (u64)(x - (s << ii.segshift)) * e.slope) >> 32);
    return k < ii.nb ? k : ii.nb - 1;
}
// Smallest relative value that falls in bin k or later (k < nb).
__device__ __forceinline__ u64 fine_bin_start(u32 k, const InstInfo& ii, const SegEntry* tab)
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

// ---------------------------------------------------------------------------
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
    int lo = 0, hi = R;
    while (lo < hi) {
        int m = (lo + hi) >> 1;
        if (row[m] <= v) lo = m + 1; else hi = m;
    }
    return lo;
}

// The same for row p of stored (inst != nullptr) or predicted rows.
__device__ __forceinline__ int zl_iters_of(const i64* inst, const i64* le, const i64* iv, int p, int R, i64 v)
{
    if (inst) return zl_iters(inst + (size_t)p * R, R, v);
    const i64 l = le[p], s = iv[p];
    int lo = 0, hi = R;
    while (lo < hi) {
        const int m = (lo + hi) >> 1;
        if ((i64)((u64)l + (u64)(m + 1) * (u64)s) <= v) lo = m + 1; else hi = m;
    }
    return lo;
}

// ---------------------------------------------------------------------------
// Window workgroup: LDS layout and the sort/scan/argmin steps.
//
// A record is (key: low 32 bits, delta: high 32 bits).  Keys are relative to
// the window start and windows are at most 2^32 wide.  Deltas fit 32 bits when
// the instance's range does; otherwise (WIDE) the upper half of each delta
// lives in a second plane and a window holds half as many records.  Record q
// lives at slot q + (q >> 4): one pad slot per 16 records keeps both the
// wave-striped access of the sort and the blocked access of the scan free of
// bank conflicts.
template <int NT, int ITEMS>
struct WinCfg {
    static constexpr int NW = NT / WAVE;
    static constexpr int CAP = NT * ITEMS;
    static constexpr int DB_MAX = NT >= 256 ? 8 : 6;     // widest radix digit (one thread per digit value)
    static constexpr int RADIX_MAX = 1 << DB_MAX;
    static constexpr int RECS = CAP + CAP / 16 + 2;
    static constexpr int CAP_WIDE = CAP / 2 > 0 ? CAP / 2 : 1;
    static constexpr int ITEMS_WIDE = ITEMS / 2 > 0 ? ITEMS / 2 : 1;
    static constexpr int RECS_WIDE = NT * ITEMS_WIDE + NT * ITEMS_WIDE / 16 + 2;
    static constexpr size_t REC_BYTES = (size_t)RECS * 8 > (size_t)RECS_WIDE * 12 ? (size_t)RECS * 8 : (size_t)RECS_WIDE * 12;
    static constexpr int CNT_WORDS = (NW * RADIX_MAX > 2 * NT) ? NW * RADIX_MAX : 2 * NT;
    static constexpr int RED_WORDS = 3 * NW + 8;          // u64 scratch for scans and reductions
    static constexpr size_t BYTES = (REC_BYTES + 15) / 16 * 16 + (size_t)RED_WORDS * 8 + (size_t)CNT_WORDS * 4;
};

struct Smem {       // carved from one static LDS array
    u64* recs;      // record plane
    u32* dhi;       // upper halves of the deltas (WIDE only)
    u64* red;       // reduction scratch
    u32* cnt;       // per-wave digit counters; row offsets while loading
};

template <int NT, int ITEMS>
__device__ __forceinline__ Smem carve(unsigned char* smem)
{
    using C = WinCfg<NT, ITEMS>;
    Smem s;
    s.recs = (u64*)smem;
    s.dhi = (u32*)(s.recs + C::RECS_WIDE);
    s.red = (u64*)(smem + (C::REC_BYTES + 15) / 16 * 16);
    s.cnt = (u32*)(s.red + C::RED_WORDS);
    return s;
}

__device__ __forceinline__ int phys(int q) { return q + (q >> 4); }

// Lanes of this wave whose digit equals mine.
__device__ __forceinline__ u64 match_digit(u32 d, int dbits)
{
    u64 peers = ~0ull;
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        if (b < dbits) {
            const bool bit = (d >> b) & 1u;
            const u64 bal = __ballot(bit);
            peers &= bit ? bal : ~bal;
        }
    }
    return peers;
}

// zl_sort: stable LSD radix sort of records [0, NT*items) by the low `kbits`
// bits of the key.  Wave w owns positions [w*64*items, (w+1)*64*items); in
// round j lane l holds position w*64*items + j*64 + l.  Ranks within a wave
// come from ballots, per-wave digit counts live in cnt[w][digit]; a digit-major
// scan of those counts gives every (wave, digit) its first output position.
template <int NT, int ITEMS, bool WIDE>
__device__ __forceinline__ void zl_sort(const Smem& sm, int items, int kbits)
{
    using C = WinCfg<NT, ITEMS>;
    constexpr int IT = WIDE ? C::ITEMS_WIDE : ITEMS;
    u64* recs = sm.recs;
    u32* cnt = sm.cnt;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid >> 6;
    if (kbits <= 0) return;
    const int npass = (kbits + C::DB_MAX - 1) / C::DB_MAX;
    const int dbits = (kbits + npass - 1) / npass;
    const u32 radix = 1u << dbits, dmask = radix - 1u;
    const u64 lt = (1ull << lane) - 1ull;
    volatile u32* mycnt = cnt + wave * C::RADIX_MAX;
    const int wbase = wave * WAVE * items + lane;

    for (int pass = 0; pass < npass; ++pass) {
        const int sh = pass * dbits;
        for (u32 d = lane; d < radix; d += WAVE) mycnt[d] = 0;
        u32 key[IT], dl[IT], dh[WIDE ? IT : 1], rank[IT];
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            if (j < items) {
                const u64 r = recs[phys(wbase + j * WAVE)];
                key[j] = (u32)r;
                dl[j] = (u32)(r >> 32);
                if (WIDE) dh[j] = sm.dhi[phys(wbase + j * WAVE)];
                const u32 d = (key[j] >> sh) & dmask;
                const u64 peers = match_digit(d, dbits);
                const u32 below = __popcll(peers & lt);
                const u32 old = mycnt[d];
                if (below == 0) mycnt[d] = old + (u32)__popcll(peers);
                rank[j] = old + below;
            }
        }
        __syncthreads();
        // digit-major exclusive scan over (digit, wave)
        u32 mine = 0;
        if ((u32)tid < radix) {
#pragma unroll 4
            for (int w = 0; w < C::NW; ++w) mine += cnt[w * C::RADIX_MAX + tid];
        }
        u32 all;
        u32 run = block_excl_scan<u32, NT>(mine, (u32*)sm.red, all);
        if ((u32)tid < radix) {
#pragma unroll 4
            for (int w = 0; w < C::NW; ++w) {
                const u32 c = cnt[w * C::RADIX_MAX + tid];
                cnt[w * C::RADIX_MAX + tid] = run;
                run += c;
            }
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            if (j < items) {
                const u32 d = (key[j] >> sh) & dmask;
                const int pos = (int)(mycnt[d] + rank[j]);
                recs[phys(pos)] = (u64)key[j] | ((u64)dl[j] << 32);
                if (WIDE) sm.dhi[phys(pos)] = dh[j];
            }
        }
        __syncthreads();
    }
}

// zl_scan + zl_argmin over the sorted records [0, total).
// Thread t owns positions [t*items, (t+1)*items).  S(q) = inclusive prefix of
// the deltas; candidate at q if it ends a run of equal keys and
// a + key >= thr; value  P*key + W0 - S(q)  (all arithmetic modulo 2^64; the
// true value is in [0, 2^63) by the caller's precondition).
// Returns the block-wide first minimum: (wait, key) with wait == U64_MAX if
// there is no candidate.
template <int NT, bool WIDE>
__device__ __forceinline__ void zl_scan_argmin(const Smem& sm, int items, int total,
                                               u64 a, u64 thr, u64 P, u64 W0,
                                               u64& best_wait, u32& best_key)
{
    const u64* recs = sm.recs;
    u64* red = sm.red;
    const int tid = threadIdx.x;
    const int q0 = tid * items;
    int qe = q0 + items;
    if (qe > total) qe = total;
    u64 local = 0;
    for (int q = q0; q < qe; ++q) {
        local += recs[phys(q)] >> 32;
        if (WIDE) local += (u64)sm.dhi[phys(q)] << 32;
    }
    u64 sum_all;
    u64 S = block_excl_scan<u64, NT>(local, red, sum_all);

    u64 bw = U64_MAX;
    u32 bq = 0xffffffffu, bk = 0;
    u64 r = (q0 < qe) ? recs[phys(q0)] : 0ull;
    for (int q = q0; q < qe; ++q) {
        const u32 key = (u32)r;
        S += r >> 32;
        if (WIDE) S += (u64)sm.dhi[phys(q)] << 32;
        const bool has_next = q + 1 < total;
        const u64 rn = has_next ? recs[phys(q + 1)] : 0ull;
        const bool run_end = !has_next || (u32)rn != key;
        const bool admissible = a + key >= thr;
        if (run_end && admissible) {
            const u64 w = P * (u64)key + W0 - S;
            if (w < bw) { bw = w; bq = (u32)q; bk = key; }
        }
        r = rn;
    }
    // block arg-min over (wait, position): smaller wait, then earlier position
#pragma unroll
    for (int d = WAVE / 2; d > 0; d >>= 1) {
        const u64 ow = __shfl_xor(bw, d, WAVE);
        const u32 oq = __shfl_xor(bq, d, WAVE);
        const u32 ok = __shfl_xor(bk, d, WAVE);
        if (ow < bw || (ow == bw && oq < bq)) { bw = ow; bq = oq; bk = ok; }
    }
    constexpr int NW = NT / WAVE;
    const int lane = tid & (WAVE - 1), wave = tid >> 6;
    if (lane == 0) { red[wave] = bw; red[NW + wave] = ((u64)bq << 32) | bk; }
    __syncthreads();
    bw = red[0];
    u64 bqk = red[NW];
#pragma unroll
    for (int w = 1; w < NW; ++w) {
        const u64 ow = red[w], oqk = red[NW + w];
        if (ow < bw || (ow == bw && (u32)(oqk >> 32) < (u32)(bqk >> 32))) { bw = ow; bqk = oqk; }
    }
    __syncthreads();
    best_wait = bw;
    best_key = (u32)bqk;
}

// Sentinels behind the last record, so that whole rounds of 64 can be sorted.
template <int NT>
__device__ __forceinline__ void fill_sentinels(u64* recs, int total, int items)
{
    for (int q = total + threadIdx.x; q < NT * items; q += NT) recs[phys(q)] = 0x00000000ffffffffull;
}

// zl_delta for a value interval [a, el] (el - a < 2^32) of the rows in `rw`:
// gathers every row's segment into records (key = value - a, delta = value -
// the row's previous value, or value - a for a row's very first entry) in
// slots [0, total).  At most `cap` records are stored; the true total is
// returned.  w0 accumulates this thread's share of W0 = sum_p (a - last value
// of row p before the interval).  Rows are taken NT at a time: a block scan of
// the segment lengths gives every row its first slot, then consecutive threads
// take consecutive slots, so reads within a segment coalesce.
template <int NT, bool WIDE, bool PAD>
__device__ __forceinline__ int zl_delta(const Smem& sm, const Rows& rw, u64 a, u64 el, bool lx, bool rx,
                                        int cap, u64& w0, int& bad)
{
    const int tid = threadIdx.x;
    u32* rowoff = sm.cnt;
    u32* rowlo = sm.cnt + NT;
    int total = 0;
    for (int p0 = 0; p0 < rw.P; p0 += NT) {
        const int p = p0 + tid;
        u32 lo = 0, hi = 0;
        if (p < rw.P) {
            sub_range(rw, p, a, el, lx, rx, lo, hi);
            if (lo > 0) w0 += a - rw.rel(p, lo - 1);
        }
        u32 chunk;
        const u32 off = block_excl_scan<u32, NT>(hi - lo, (u32*)sm.red, chunk);
        rowoff[tid] = off;
        rowlo[tid] = lo;
        __syncthreads();
        const int room = cap - total;
        const int take = (int)chunk < room ? (int)chunk : room;
        const int nrows = (rw.P - p0) < NT ? (rw.P - p0) : NT;
        for (int e = tid; e < take; e += NT) {
            int l = 0, h = nrows;                 // the last row r with rowoff[r] <= e
            while (h - l > 1) {
                const int m = (l + h) >> 1;
                if (rowoff[m] <= (u32)e) l = m; else h = m;
            }
            const u32 i = rowlo[l] + ((u32)e - rowoff[l]);
            const i64 cur = rw.value(p0 + l, i);
            const u64 rel = (u64)cur - rw.base;
            u64 prel = a;
            if (i > 0) {
                const i64 prv = rw.value(p0 + l, i - 1);
                prel = (u64)prv - rw.base;
                bad |= (cur < prv);
            }
            const u64 dl = rel - prel;
            const int slot = PAD ? phys(total + e) : total + e;
            sm.recs[slot] = (u64)(u32)(rel - a) | (dl << 32);
            if (WIDE) sm.dhi[slot] = (u32)(dl >> 32);
        }
        total += (int)chunk;
        __syncthreads();
    }
    return total;
}

// ---------------------------------------------------------------------------
// Fast path of zl_sort + zl_scan + zl_argmin for one window whose keys are
// spread evenly enough: a counting sort into NB value buckets (LDS atomics; the
// order inside a bucket does not matter) followed by direct evaluation.
// With BP(b) = sum of the deltas in all buckets below b, the prefix sum at an
// element of bucket b is BP(b) + the deltas of the bucket's elements whose key
// is <= its own; equal keys get equal values, so no run-end rule is needed.
// The work is total + sum over buckets of size^2: a bucket with more than
// BUCKET_LIMIT entries makes the caller fall back to the radix sort.
// One exchange for three block-wide results: the exclusive scan of h (a packed
// count and sum: the two fields must not overflow into each other), (WITH_X) the
// sum of x and (WITH_U) the minimum over all threads of local(i) - (sum of h's low
// SUM_BITS over the waves before the thread's), where i is the inclusive scan of
// h inside the thread's wave; local(i) == INT64_MAX stands for "none".
// `red` holds 3*NT/64 u64 words; the caller must pass a barrier before it
// writes them again.
template <int NT, bool WITH_X, bool WITH_U, class Local>
__device__ __forceinline__ void block_scan_pair(u64 h, u64 x, Local local, u64* red, u64 low_mask,
                                                u64& hbase, u64& xsum, i64& umin)
{
    constexpr int NW = NT / WAVE;
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x >> 6;
    const u64 hi = wave_scan(h, OpAdd());
    if (WITH_X) x = wave_scan(x, OpAdd());
    i64 u = INT64_MAX;
    if (WITH_U) u = wave_scan((i64)local(hi), OpMin());
    if (lane == WAVE - 1) {
        red[wave] = hi;
        if (WITH_X) red[NW + wave] = x;
        if (WITH_U) red[2 * NW + wave] = (u64)u;
    }
    __syncthreads();
    u64 hb = 0, xx = 0, run = 0;
    i64 um = INT64_MAX;
#pragma unroll 2                       // more would hold all the partial results in registers at once
    for (int w = 0; w < NW; ++w) {
        const u64 xh = red[w];
        if (w < wave) hb += xh;
        if (WITH_X) xx += red[NW + w];
        if (WITH_U) {
            const i64 uw = (i64)red[2 * NW + w];
            const i64 cand = uw == INT64_MAX ? uw : uw - (i64)run;
            um = cand < um ? cand : um;
            run += xh & low_mask;
        }
    }
    hbase = hb + hi - h;
    xsum = xx;
    umin = um;
}

template <int NT, int ITEMS, bool TABLE = true>
struct HotCfg {
    static constexpr int NW = NT / WAVE;
    static constexpr int CAP = NT * ITEMS;
    static constexpr int NB = 2 * NT;                     // value buckets; each thread scans two
    static constexpr int RED_WORDS = 4 * NW + 8;
    static constexpr int COARSE = 256;                    // coarse value bins behind an equalising bucket map
    static constexpr int PAD = 4;                         // record slots after the last one that a 4-wide read may touch
    static constexpr int BSUM_AT = CAP + PAD;             // bucket words follow the records
    static constexpr size_t BYTES = (size_t)BSUM_AT * 8 + (size_t)NB * 8 + (size_t)RED_WORDS * 8 + (size_t)NB * 4 +
                                    (TABLE ? (size_t)COARSE * 16 : 0);  // the coarse tables are the last area
};
// One LDS word per bucket holds its entry count (upper bits) and the sum of its
// deltas (lower SUM_BITS bits: at most 16384 deltas below 2^32 each).
constexpr int SUM_BITS = 46;
constexpr u64 SUM_MASK = (1ull << SUM_BITS) - 1;
constexpr u32 BUCKET_LIMIT = 64;
constexpr int GATHER_BATCH = 8;           // elements a thread loads before it uses any of them
constexpr int GATHER_TAIL = 8;            // the same beyond the first batch

template <int NT, int ITEMS>
__device__ __forceinline__ Smem carve_hot(unsigned char* smem)
{
    using H = HotCfg<NT, ITEMS>;
    Smem s;
    s.recs = (u64*)smem;
    s.dhi = nullptr;
    s.red = s.recs + H::BSUM_AT + H::NB;      // bucket sums sit between the records and the scratch
    s.cnt = (u32*)(s.red + H::RED_WORDS);
    return s;
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
    __device__ __forceinline__ u32 operator()(u32 key) const
    {
        const u32 b = (u32)(((u64)key * scale) >> 32);
        return b < top ? b : top;
    }
    // lo <= every key of bucket b <= hi (for keys within [0, span]).  A key k of bucket
    // b < top has b * 2^32 <= k * scale < (b + 1) * 2^32; inv52 is at most one short of
    // 2^52 / scale, which costs less than 2 after the shift (b + 1 <= 2^11).
    __device__ __forceinline__ void bounds(u32 b, u32& lo, u32& hi) const
    {
        const u64 l = ((u64)b * inv52) >> 20;
        const u64 h = (((u64)(b + 1) * inv52) >> 20) + 2;
        hi = (b >= top || h > span) ? span : (u32)h;
        lo = l > hi ? hi : (u32)l;
    }
    // The same for buckets b and b + 1 with one product: floor((b + 1) * x) >= floor(b * x) +
    // floor(x), and a bucket is less than floor(x) + 2 wide (x = inv52 / 2^20).
    __device__ __forceinline__ void bounds_pair(u32 b, u32& lo0, u32& hi0, u32& lo1, u32& hi1) const
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
__device__ __forceinline__ u32 linear_scale(u64 span, u32 nb)
{
    const u64 q = ((u64)nb << 32) / (span + 1);
    return q >= 0xffffffffull ? 0xffffffffu : (q ? (u32)q : 1u);
}
__device__ __forceinline__ LinearMap linear_map(u32 span, u32 nb, u32 scale, u64 inv52)
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
    __device__ __forceinline__ u32 coarse(u32 key) const { const u32 c = key >> cshift; return c < 255u ? c : 255u; }
    __device__ __forceinline__ u32 operator()(u32 key) const
    {
        const u64 e = tab[coarse(key)];
        return (u32)e + (u32)(((u64)(key & cmask) * (e >> 32)) >> 32);
    }
    // lo <= every key of bucket b <= hi.  The bins that reach bucket b are consecutive:
    // the lower bound comes from the first of them, the upper bound from the last; inside
    // a bin the bucket is linear in the key's low bits, as for LinearMap.
    __device__ __forceinline__ void bounds(u32 b, u32& lo, u32& hi) const
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
    __device__ __forceinline__ void bounds_pair(u32 b, u32& lo0, u32& hi0, u32& lo1, u32& hi1) const
    {
        bounds(b, lo0, hi0);
        bounds(b + 1, lo1, hi1);
    }
};

// The records of a window, held ITEMS per thread in registers (item j of thread t
// is record j*NT + t, present if that is below `total`) -> first minimum
// (wait, key) of P*key + W0 - S(key) over keys with a + key >= thr, W0 being the
// block sum of `w0` (taken as 0 unless WITH_W0).
// On entry the bucket words must be zero and a barrier must have passed since;
// the record area may hold anything (it is overwritten).  On return some threads
// may still be reading LDS: the caller passes a barrier before writing it again.
// Returns false (nothing computed) if some bucket is over the limit.
template <int NT, int ITEMS, bool WITH_W0, class Map>
__device__ __forceinline__ bool zl_bucket_finish(const Smem& sm, const u32 (&key)[ITEMS], const u32 (&dl)[ITEMS],
                                                 const Map bucket, int total, u64 a, u64 thr, u32 P, u64 w0,
                                                 u64& best_wait, u32& best_key)
{
    using H = HotCfg<NT, ITEMS>;
    u64* recs = sm.recs;
    u64* bsum = sm.recs + H::BSUM_AT;
    u32* cnt = sm.cnt;
    const int tid = threadIdx.x;
    u32* live_count = (u32*)(sm.red + H::RED_WORDS - 1);              // entries of the compact list
    u32* deep = live_count + 1;                                       // set if some bucket is over the limit
    if (tid == 0) { *live_count = 0; *deep = 0; }
    // zl_sort, step 1: per bucket, entry count and sum of deltas in one word
#pragma unroll
    for (int j = 0; j < ITEMS; ++j)
        if (j * NT + tid < total) {
            const u32 bid = bucket(key[j]);
            atomicAdd(&bsum[bid], (1ull << SUM_BITS) | (u64)dl[j]);
        }
    __syncthreads();
    // step 2: exclusive scans over the buckets (two per thread)
    const u64 h0 = bsum[2 * tid], h1 = bsum[2 * tid + 1];
    const u32 c0 = (u32)(h0 >> SUM_BITS), c1 = (u32)(h1 >> SUM_BITS);
    const u64 s0 = h0 & SUM_MASK, s1 = h1 & SUM_MASK;
    constexpr bool PRUNE = Map::HAS_BOUNDS;
    constexpr u32 DROPPED = 0x80000000u;
    // Most buckets cannot hold the minimum.  With E = the sum of deltas up to the end
    // of bucket b and lo <= keys of b <= hi: the bucket's largest key kmax is a
    // candidate with wait P*kmax + W0 - E <= P*hi + W0 - E =: ub(b) (if the whole
    // bucket is admissible), and every key of b waits at least P*lo + W0 - E =: lb(b).
    // Buckets with lb(b) above the smallest ub are dropped; the others get room in a
    // compact list (in any order) and only their entries are scattered and evaluated.
    u32 lo0 = 0, hi0 = 0, lo1 = 0, hi1 = 0;
    const u64 need = thr > a ? thr - a : 0;                           // keys >= need are admissible
    if (PRUNE) bucket.bounds_pair(2 * tid, lo0, hi0, lo1, hi1);
    // smallest P*hi - E over the thread's admissible buckets, E counted from the wave's first bucket
    auto local_bound = [&](u64 incl) {
        const u64 e1 = incl & SUM_MASK;
        i64 u = INT64_MAX;
        if (c0 && lo0 >= need) u = (i64)((u64)P * hi0 - (e1 - s1));
        if (c1 && lo1 >= need) { const i64 u1 = (i64)((u64)P * hi1 - e1); u = u1 < u ? u1 : u; }
        return u;
    };
    u64 hbase, W0;
    i64 ubmin;
    if ((c0 > c1 ? c0 : c1) > BUCKET_LIMIT) *deep = 1;
    block_scan_pair<NT, WITH_W0, PRUNE>(h0 + h1, w0, local_bound, sm.red, SUM_MASK, hbase, W0, ubmin);
    if (*deep) return false;
    const u32 cbase = (u32)(hbase >> SUM_BITS);
    const u64 sbase = hbase & SUM_MASK;
    u64 bw = U64_MAX;
    u32 bk = 0xffffffffu;
    if constexpr (PRUNE) {
        const u64 e0 = sbase + s0, e1 = e0 + s1;
        const i64 ub0 = (i64)((u64)P * hi0 - e0), ub1 = (i64)((u64)P * hi1 - e1);       // both without W0, like ubmin
        // (a bucket whose keys are all below `need` holds no candidate at all)
        const bool live0 = c0 && hi0 >= need && ub0 - (i64)((u64)P * (hi0 - lo0)) <= ubmin;
        const bool live1 = c1 && hi1 >= need && ub1 - (i64)((u64)P * (hi1 - lo1)) <= ubmin;
        u32 at0 = DROPPED, at1 = DROPPED;
        if (live0) at0 = atomicAdd(live_count, c0);
        if (live1) at1 = atomicAdd(live_count, c1);
        cnt[2 * tid] = at0; cnt[2 * tid + 1] = at1;
        bsum[2 * tid] = sbase | ((u64)(at0 & (DROPPED - 1)) << SUM_BITS);     // BP(bucket) and the bucket's first slot
        bsum[2 * tid + 1] = e0 | ((u64)(at1 & (DROPPED - 1)) << SUM_BITS);
        __syncthreads();
        // step 3: scatter the entries of the live buckets; afterwards cnt[b] is the end of bucket b
#pragma unroll
        for (int j = 0; j < ITEMS; ++j)
            if (j * NT + tid < total) {
                const u32 bid = bucket(key[j]);
                const u32 slot = atomicAdd(&cnt[bid], 1u);
                if (slot < DROPPED) recs[slot] = (u64)key[j] | ((u64)dl[j] << 32);
            }
        __syncthreads();
        const int live = (int)*live_count;
        // zl_scan + zl_argmin: every listed entry evaluates its own candidate
        for (int q = tid; q < live; q += NT) {
            const u32 k = (u32)recs[q];
            const u32 bid = bucket(k);
            const u32 e = cnt[bid];
            const u64 hb = bsum[bid];
            u32 x = (u32)(hb >> SUM_BITS);
            u64 S = hb & SUM_MASK;
            for (; x < e; ++x) {
                const u64 r = recs[x];
                S += ((u32)r <= k) ? r >> 32 : 0ull;
            }
            if ((u64)k >= need) {
                const u64 w = (u64)P * k + W0 - S;
                if (w < bw || (w == bw && k < bk)) { bw = w; bk = k; }
            }
        }
    } else {
    cnt[2 * tid] = cbase; cnt[2 * tid + 1] = cbase + c0;
    bsum[2 * tid] = sbase | ((u64)cbase << SUM_BITS);                 // BP(bucket) and the bucket's first slot
    bsum[2 * tid + 1] = (sbase + s0) | ((u64)(cbase + c0) << SUM_BITS);
    __syncthreads();
    // step 3: scatter; afterwards cnt[b] is the end of bucket b
#pragma unroll
    for (int j = 0; j < ITEMS; ++j)
        if (j * NT + tid < total) {
            const u32 bid = bucket(key[j]);
            const u32 slot = atomicAdd(&cnt[bid], 1u);
            recs[slot] = (u64)key[j] | ((u64)dl[j] << 32);
        }
    // a 4-wide read of the last bucket may run past the end: entries that add nothing
    if (tid < H::PAD - 1) recs[total + tid] = 0xffffffffull;
    __syncthreads();
    // zl_scan + zl_argmin: every element evaluates its own candidate.  The bucket map
    // is monotone, so whatever a 4-wide read picks up beyond the element's own bucket
    // has a larger key and drops out by the same comparison.
    for (int q = tid; q < total; q += NT) {
        const u32 k = (u32)recs[q];
        const u32 bid = bucket(k);
        const u32 e = cnt[bid];
        const u64 hb = bsum[bid];
        u32 x = (u32)(hb >> SUM_BITS);
        u64 S = hb & SUM_MASK;
        for (; x < e; x += 4) {                       // four entries per trip: one LDS round trip, not four
            const u64 r0 = recs[x], r1 = recs[x + 1], r2 = recs[x + 2], r3 = recs[x + 3];
            S += ((u32)r0 <= k) ? r0 >> 32 : 0ull;
            S += ((u32)r1 <= k) ? r1 >> 32 : 0ull;
            S += ((u32)r2 <= k) ? r2 >> 32 : 0ull;
            S += ((u32)r3 <= k) ? r3 >> 32 : 0ull;
        }
        if (a + k >= thr) {
            const u64 w = (u64)P * k + W0 - S;
            if (w < bw || (w == bw && k < bk)) { bw = w; bk = k; }
        }
    }
    }
    // block arg-min over (wait, key): smaller wait, then smaller key
    wave_argmin(bw, bk);
    constexpr int NW = NT / WAVE;
    const int lane = tid & (WAVE - 1), wave = tid >> 6;
    u64* red = sm.red;
    if (lane == WAVE - 1) { red[wave] = bw; red[NW + wave] = bk; }
    __syncthreads();
    bw = red[0];
    bk = (u32)red[NW];
#pragma unroll
    for (int w = 1; w < NW; ++w) {
        const u64 ow = red[w];
        const u32 ok = (u32)red[NW + w];
        if (ow < bw || (ow == bw && ok < bk)) { bw = ow; bk = ok; }
    }
    best_wait = bw;                       // the caller passes a barrier before LDS is written again
    best_key = bk;
    return true;
}

// zl_delta for the fast window path: the rows' index ranges are exactly the
// window (no searching), every value of the instance fits 32 bits relative to
// its base, and byte offsets into the instance fit 32 bits.  Two sweeps:
//   1. one thread per row (a round covers 1024 rows): segment lengths, one block
//      scan for the first slots, and a source word for every element of a
//      segment written into that element's slot (index into the instance;
//      FIRST_OF_ROW: the row's very first entry, which has no predecessor;
//      FIRST_OF_SEGMENT: the entry whose predecessor lies before the window).
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
constexpr u64 FIRST_OF_ROW = 1ull << 32, FIRST_OF_SEGMENT = 1ull << 33;
constexpr int PRED_ROW_SHIFT = 34;        // predicted rows: the row number sits above the two flags
// rows a thread takes per round of sweep 1: one round covers 1024 rows
template <int NT> constexpr int ROWS_PER_THREAD = NT >= 1024 ? 1 : 1024 / NT;
constexpr int WINDOWS_PER_BLOCK = 2;      // consecutive windows a workgroup handles, one after the other
constexpr u64 HOT_MAX_ENTRIES = 1ull << 29;   // P*R below this: byte offsets into an instance fit 32 bits

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
    u64 src[G];
    u32 cur[G], prv[G];
#pragma unroll
    for (int j = 0; j < G; ++j) {
        const int q = (g + j) * NT + tid;
        src[j] = q < total ? recs[q] : FIRST_OF_ROW;               // beyond the end: entry 0, harmless
    }
#pragma unroll
    for (int j = 0; j < G; ++j) {
        if (PRED) {
            // predicted rows: the source word holds the row (above the flags) and the index in it
            const uint2 fs = par[(u32)(src[j] >> PRED_ROW_SHIFT)];  // first value of the row, interval
            cur[j] = fs.x + (u32)src[j] * fs.y;
            prv[j] = cur[j] - fs.y;
        } else {
            const u32 at = (u32)src[j];
            const u32 pat = at - (1u - ((u32)(src[j] >> 32) & 1u));    // a row's first entry stands in for its predecessor
            cur[j] = *(const u32*)(bytes + (at << 3));
            prv[j] = *(const u32*)(bytes + (pat << 3));
        }
    }
#pragma unroll
    for (int j = 0; j < G; ++j) {
        const u32 from = (src[j] & FIRST_OF_ROW) ? start : prv[j];
        key[g + j] = cur[j] - start;
        dl[g + j] = cur[j] - from;
        w0 += (src[j] & FIRST_OF_SEGMENT) ? (u64)(start - from) : 0ull;   // below 2^32 like every relative value
    }
}

// Sweep 1 of the window gather (see above): a source word for every entry of the window in
// its slot.  Returns the number of entries (slots beyond `cap` are not written).  For the rows
// without an entry in the window the distances from their last value before it to the window
// start are summed into before_sum and their maximum goes to before_max.  WITH_LAST marks a
// row's very last entry too (stored rows only: the mark shares its bit with the row number).
constexpr u64 LAST_OF_ROW = 1ull << 34;
template <int NT, class CT, bool PRED, bool WITH_LAST>
__device__ __forceinline__ int zl_place_rows(const Smem& sm, const Rows& rw, u32 start, int cap,
                                             const u32 (&lo0)[ROWS_PER_THREAD<NT>], const u32 (&hi0)[ROWS_PER_THREAD<NT>],
                                             u64& before_sum, u32& before_max)
{
    static_assert(!(PRED && WITH_LAST), "the last-of-row mark is for stored rows");
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
                else before[c] = *(const u32*)(bytes + (((u32)p * (u32)rw.R + lo[c] - 1u) << 3));
            }
        }
        u32 round;
        u32 slot = (u32)total + block_excl_scan<u32, NT>(mine, (u32*)sm.red, round);
#pragma unroll
        for (int c = 0; c < RPT; ++c) {
            const int p = p0 + c * NT + tid;
            if (p < rw.P) {
                const u64 row = PRED ? (u64)(u32)p << PRED_ROW_SHIFT : 0ull;
                u64 src = row | (u64)(PRED ? lo[c] : (u32)p * (u32)rw.R + lo[c]) | FIRST_OF_SEGMENT |
                          (lo[c] == 0 ? FIRST_OF_ROW : 0ull);
                for (u32 i = lo[c]; i < hi[c] && slot < (u32)cap; ++i, ++slot) {
                    recs[slot] = (WITH_LAST && i + 1 == (u32)rw.R) ? (src | LAST_OF_ROW) : src;
                    src = row | (u64)((u32)src + 1u);
                }
            }
        }
#pragma unroll
        for (int c = 0; c < RPT; ++c) {                      // below 2^32 like every relative value
            const u32 gone = start - before[c];
            before_sum += (u64)gone;
            before_max = gone > before_max ? gone : before_max;
        }
        total += (int)round;
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
    const int total = zl_place_rows<NT, CT, PRED, false>(sm, rw, start, cap, lo0, hi0, w0, unused);
    if (total > cap) return total;

    constexpr int G0 = ITEMS < GATHER_BATCH ? ITEMS : GATHER_BATCH;
    gather_batch<NT, ITEMS, G0, PRED>(recs, bytes, rw.par, 0, total, start, key, dl, w0);
    static_assert((ITEMS - G0) % GATHER_TAIL == 0 || ITEMS < GATHER_BATCH, "tail batches must tile the items");
#pragma unroll
    for (int g = G0; g < ITEMS; g += GATHER_TAIL)
        gather_batch<NT, ITEMS, GATHER_TAIL, PRED>(recs, bytes, rw.par, g, total, start, key, dl, w0);
    return total;
}

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
// most 2^32 wide and holds at most `cap` entries and is handled in one go.
// Otherwise it is walked in pieces that do fit, cut by bisection on the value;
// a single value that alone occurs more than `cap` times is one candidate and
// is evaluated directly from the rows.  (bw, bb) is updated with the first
// minimum found: smaller wait, then smaller barrier (relative to base).
template <int NT, int ITEMS, bool WIDE>
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
        if (el - a > 0xffffffffull) { el = a + 0xffffffffull; rx = false; }
        u64 w0 = 0;
        int total = zl_delta<NT, WIDE, true>(sm, rw, a, el, lx, rx, CAPW, w0, bad);
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
                total = zl_delta<NT, WIDE, true>(sm, rw, a, el, lx, false, CAPW, w0, bad);
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
            const u64 W0 = block_reduce<u64, NT>(w0, sm.red, OpAdd());   // also orders the record writes
            zl_sort<NT, ITEMS, WIDE>(sm, items, bit_length(el - a));
            u64 w;
            u32 key;
            zl_scan_argmin<NT, WIDE>(sm, items, total, a, thr, (u64)rw.P, W0, w, key);
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

// ---------------------------------------------------------------------------
// One workgroup per instance (P*R <= NT*ITEMS): the whole search in LDS.
template <int NT, int ITEMS, bool PRED>        // PRED: rows are le[p] + (i + 1) * iv[p] instead of stored
__global__ __launch_bounds__(NT) void zl_instance_kernel(
    const i64* __restrict__ ts, const i64* __restrict__ le, const i64* __restrict__ iv, int P, int R, int rshift,
    i64* __restrict__ barrier, int* __restrict__ iters, i64* __restrict__ wait,
    int* __restrict__ status)
{
    using H = HotCfg<NT, ITEMS>;
    __shared__ __align__(16) unsigned char smem[H::BYTES];
    const Smem sm = carve_hot<NT, ITEMS>(smem);

    const int tid = threadIdx.x;
    const i64 b = blockIdx.x;
    const int n = P * R;
    const i64* __restrict__ inst = PRED ? nullptr : ts + b * (i64)n;
    const i64* __restrict__ lep = PRED ? le + b * (i64)P : nullptr;
    const i64* __restrict__ ivp = PRED ? iv + b * (i64)P : nullptr;
    auto at = [&](int e) -> i64 {                       // element e of the instance
        if (!PRED) return inst[e];
        const int p = rshift >= 0 ? (e >> rshift) : (e / R);
        return (i64)((u64)lep[p] + (u64)(e - p * R + 1) * (u64)ivp[p]);
    };

    // zl_delta.  Every element is loaded once, all loads of a thread in flight
    // together: wave w takes elements [w*64*items, (w+1)*64*items), 64 consecutive
    // ones per round, so the previous element sits in the neighbouring lane.
    // The instance minimum is not known yet, so keys are first taken relative to
    // the instance's first element t00 (mod 2^32) and shifted afterwards.
    {
        u64* bsum = sm.recs + H::BSUM_AT;
        bsum[tid] = 0; bsum[tid + NT] = 0;
    }
    const int lane = tid & (WAVE - 1), wave = tid >> 6;
    const int items = (n + NT - 1) / NT;
    const int wbase = wave * WAVE * items;
    const i64 t00 = at(0);
    i64 v[ITEMS];
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const int e = wbase + j * WAVE + lane;
        v[j] = (j < items && e < n) ? at(e) : 0;
    }
    i64 carry = (wbase > 0 && wbase < n) ? at(wbase - 1) : 0;   // element ahead of the wave's first
    i64 mn = INT64_MAX, mxf = INT64_MIN, mxl = INT64_MIN;         // min first, max first, max last of the rows
    int bad = 0;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const int e = wbase + j * WAVE + lane;
        i64 prv = __shfl_up(v[j], 1, WAVE);
        if (lane == 0) prv = carry;
        carry = __shfl(v[j], WAVE - 1, WAVE);
        if (j < items && e < n) {
            const int i = rshift >= 0 ? (e & (R - 1)) : (e % R);
            const u32 rel = (u32)((u64)v[j] - (u64)t00);
            u32 dl = rel;                                          // a row's first entry: completed below
            if (i == 0) { mn = v[j] < mn ? v[j] : mn; mxf = v[j] > mxf ? v[j] : mxf; }
            else { dl = (u32)((u64)v[j] - (u64)prv); bad |= (v[j] < prv); }
            if (i == R - 1) mxl = v[j] > mxl ? v[j] : mxl;
            sm.recs[e] = (u64)rel | ((u64)dl << 32);
        }
    }
    i64 base, first_max, last_max;
    block_bounds<NT>(mn, mxf, mxl, (i64*)sm.red, base, first_max, last_max);   // also orders the record writes
    const u64 range = (u64)last_max - (u64)base;
    const u64 thr = (u64)first_max - (u64)base;
    const u32 shift = (u32)((u64)t00 - (u64)base);                 // key relative to base = stored key + shift

    u32 flags = 0;
    if (range > (u64)INT64_MAX / (u64)P) flags |= EBSP_STATUS_OVERFLOW;

    if (range >> 32) {
        // deltas need more than 32 bits: left to zl_instance_general_kernel
        if (tid == 0) wait[b] = DEFERRED;
        return;
    }
    // a row's first delta is its key relative to base
    for (int p = tid; p < P; p += NT) {
        const u64 r = sm.recs[(size_t)p * R];
        sm.recs[(size_t)p * R] = (u64)(u32)r | ((u64)((u32)(r >> 32) + shift) << 32);
    }
    if (__syncthreads_or(bad)) flags |= EBSP_STATUS_UNSORTED;
    // the records go to registers for the bucket search (which reuses the record area)
    u32 key[ITEMS], dl[ITEMS];
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const int q = j * NT + tid;
        if (q < n) {
            const u64 r = sm.recs[q];
            key[j] = (u32)r + shift;
            dl[j] = (u32)(r >> 32);
        }
    }
    // the equalising bucket map: key counts of up to 256 coarse bins -> buckets per bin
    u32* coarse = sm.cnt;                                   // free until the bucket scan
    u64* tab = (u64*)(sm.cnt + H::NB);
    const int bl = bit_length(range);
    TableMap<(ITEMS >= 8)> bucket;                          // small instances: finding the bounds costs more than it saves
    bucket.tab = tab;
    bucket.cshift = bl > 8 ? (u32)(bl - 8) : 0u;
    bucket.cmask = (1u << bucket.cshift) - 1u;
    bucket.span = (u32)range;
    constexpr int CPT = H::COARSE / NT > 1 ? H::COARSE / NT : 1;      // coarse bins per thread
    for (int c = tid; c < H::COARSE; c += NT) coarse[c] = 0;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < ITEMS; ++j)
        if (j * NT + tid < n) atomicAdd(&coarse[bucket.coarse(key[j])], 1u);
    __syncthreads();
    {
        u32 c[CPT], mine = 0;
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            c[i] = tid * CPT + i < H::COARSE ? coarse[tid * CPT + i] : 0u;
            mine += c[i];
        }
        u32 all;
        u32 below_c = block_excl_scan<u32, NT>(mine, (u32*)sm.red, all);
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            if (tid * CPT + i < H::COARSE) {
                const u32 first = (u32)((u64)below_c * H::NB / (u32)n);
                u32 last = (u32)((u64)(below_c + c[i]) * H::NB / (u32)n);    // first bucket of the next coarse bin
                if (last > (u32)H::NB - 1) last = H::NB - 1;
                u32 nbk = last >= first ? last - first + 1 : 1;                // buckets this bin spreads over
                if (bucket.cshift < 32 && nbk > (1u << bucket.cshift)) nbk = 1u << bucket.cshift;
                const u64 mult = bucket.cshift ? ((u64)nbk << (32 - bucket.cshift)) - 1 : 0ull;
                tab[tid * CPT + i] = (u64)(first < (u32)H::NB ? first : (u32)H::NB - 1) | (mult << 32);
                tab[H::COARSE + tid * CPT + i] = ((u64)nbk << 52) | (mult ? (1ull << 52) / mult : 0ull);
            }
            below_c += c[i];
        }
    }
    __syncthreads();
    u64 best_wait;
    u32 bkey;
    if (!zl_bucket_finish<NT, ITEMS, false>(sm, key, dl, bucket, n, 0ull, thr, (u32)P, 0ull, best_wait, bkey)) {
        if (tid == 0) wait[b] = DEFERRED;      // clustered values: left to zl_instance_general_kernel
        return;
    }
    const i64 bar = (i64)((u64)base + bkey);
    if (tid == 0) {
        barrier[b] = bar;
        wait[b] = (i64)best_wait;
        if (status) status[b] = (int)flags;
    }
    for (int p = tid; p < P; p += NT)
        iters[b * (i64)P + p] = zl_iters_of(inst, lep, ivp, p, R, bar);
}

// The instances zl_instance_kernel deferred (value spread of 2^32 or more, or
// values too clustered for the bucket search): the general window search over
// whole rows.  A small fixed grid; every workgroup looks through its share of
// wait[] for deferred marks and handles the marked instances one after the other.
template <int NT, int ITEMS>
__global__ __launch_bounds__(NT) void zl_instance_general_kernel(
    const i64* __restrict__ ts, const i64* __restrict__ le, const i64* __restrict__ iv, i64 B, int P, int R,
    i64* __restrict__ barrier, int* __restrict__ iters, i64* __restrict__ wait,
    int* __restrict__ status)
{
    using C = WinCfg<NT, ITEMS>;
    __shared__ __align__(16) unsigned char smem[C::BYTES];
    const Smem sm = carve<NT, ITEMS>(smem);
    const int tid = threadIdx.x;
    const u32 total = (u32)B;
    const u32 share = (total + gridDim.x - 1) / gridDim.x;
    const u32 first = blockIdx.x * share;
    const u32 end = first + share < total ? first + share : total;

    for (u32 base0 = first; base0 < end; base0 += NT) {
        const u32 idx = base0 + tid;
        bool mine = idx < end && wait[idx] == DEFERRED;
        for (;;) {
            const u32 b = block_reduce<u32, NT>(mine ? idx : 0xffffffffu, (u32*)sm.red, OpMin());
            if (b == 0xffffffffu) break;
            if (b == idx) mine = false;
            const i64* __restrict__ inst = ts ? ts + (i64)b * P * R : nullptr;
            Rows ends;                            // only to read the rows' first and last entries
            ends.inst = inst; ends.le = le ? le + (i64)b * P : nullptr; ends.iv = iv ? iv + (i64)b * P : nullptr;
            ends.R = R;
            i64 mn = INT64_MAX, mxf = INT64_MIN, mxl = INT64_MIN;
            for (int p = tid; p < P; p += NT) {
                const i64 f = ends.value(p, 0), l = ends.value(p, (u32)R - 1);
                mn = f < mn ? f : mn;
                mxf = f > mxf ? f : mxf;
                mxl = l > mxl ? l : mxl;
            }
            i64 base, first_max, last_max;
            block_bounds<NT>(mn, mxf, mxl, (i64*)sm.red, base, first_max, last_max);
            const u64 range = (u64)last_max - (u64)base;
            const u64 thr = (u64)first_max - (u64)base;
            u32 flags = 0;
            if (range > (u64)INT64_MAX / (u64)P) flags |= EBSP_STATUS_OVERFLOW;

            Rows rw;
            rw.inst = inst; rw.le = le ? le + (i64)b * P : nullptr; rw.iv = iv ? iv + (i64)b * P : nullptr;
            rw.P = P; rw.R = R; rw.base = (u64)base;
            rw.cr = nullptr; rw.narrow = false; rw.stride = 0; rw.k0 = rw.k1 = 0;
            int bad = 0;
            u64 best_wait = U64_MAX, best_rel = 0;
            // the 64-bit-delta form serves every deferred instance, narrow ones included
            zl_window<NT, ITEMS, true>(sm, rw, thr, 0ull, range, best_wait, best_rel, bad);
            if (__syncthreads_or(bad)) flags |= EBSP_STATUS_UNSORTED;
            const i64 bar = (i64)((u64)base + best_rel);
            if (tid == 0) {
                barrier[b] = bar;
                wait[b] = (i64)best_wait;
                if (status) status[b] = (int)flags;
            }
            for (int p = tid; p < P; p += NT)
                iters[(i64)b * P + p] = zl_iters_of(inst, ends.le, ends.iv, p, R, bar);
        }
    }
}

// ---------------------------------------------------------------------------
// Multi-window path.

// zl_bounds: per-instance base, range, thr and the fine-bin grid.
template <int NT>
__global__ __launch_bounds__(NT) void zl_bounds_kernel(
    const i64* __restrict__ ts, const i64* __restrict__ le, const i64* __restrict__ iv, int P, int R, int bins,
    InstInfo* __restrict__ info, SegEntry* __restrict__ segtab, uint2* __restrict__ rowpar, int* __restrict__ status)
{
    static_assert(NT >= SEGS, "one thread per segment");
    __shared__ i64 red[NT / WAVE];
    __shared__ u64 seg_part[SEGS];        // entries of rows that begin or end in a segment (x 2^16)
    __shared__ u64 seg_diff[SEGS + 1];    // difference array: entries per segment of the rows that cover it whole (x 2^16)
    __shared__ u64 seg_est[SEGS];
    __shared__ u64 seg_step[SEGS];
    __shared__ u32 seg_slope[SEGS];
    const int tid = threadIdx.x;
    const i64 b = blockIdx.x;
    Rows ends;                                        // only to read the rows' first and last entries
    ends.inst = ts ? ts + b * (i64)P * R : nullptr;
    ends.le = le ? le + b * (i64)P : nullptr;
    ends.iv = iv ? iv + b * (i64)P : nullptr;
    ends.R = R;
    i64 mn = INT64_MAX, mxf = INT64_MIN, mxl = INT64_MIN;
    int backwards = 0;
    for (int p = tid; p < P; p += NT) {
        const i64 f = ends.value(p, 0), l = ends.value(p, (u32)R - 1);
        mn = f < mn ? f : mn;
        mxf = f > mxf ? f : mxf;
        mxl = l > mxl ? l : mxl;
        if (!ends.inst && R > 1 && ends.iv[p] < 0) backwards = 1;     // predicted rows: a negative interval
    }
    if (tid < SEGS) { seg_part[tid] = 0; seg_diff[tid] = 0; }
    if (tid == 0) seg_diff[SEGS] = 0;
    const i64 base = block_reduce<i64, NT>(mn, red, OpMin());
    const i64 first_max = block_reduce<i64, NT>(mxf, red, OpMax());
    const i64 last_max = block_reduce<i64, NT>(mxl, red, OpMax());
    backwards = __syncthreads_or(backwards);
    if (rowpar)                                       // predicted rows, for the window gather: low words of the first value and the interval
        for (int p = tid; p < P; p += NT)
            rowpar[b * (i64)P + p] = make_uint2((u32)(u64)ends.value(p, 0), (u32)ends.iv[p]);
    InstInfo ii;
    ii.base = base;
    ii.range = (u64)last_max - (u64)base;
    ii.thr = (u64)first_max - (u64)base;
    ii.nwin = 0;
    ii.flags = backwards ? (u32)EBSP_STATUS_UNSORTED : 0u;
    ii.pad_ = 0;
    if (ii.range > (u64)INT64_MAX / (u64)P) ii.flags |= EBSP_STATUS_OVERFLOW;
    if (backwards) ii.range = 0;                      // nothing downstream may rely on such rows
    const int bl = bit_length(ii.range);
    ii.wshift = bl > 32 ? (u32)(bl - 32) : 0u;
    const u64 top = ii.range >> ii.wshift;            // x = v >> wshift runs over [0, top], top < 2^32
    const int tl = bit_length(top);
    ii.segshift = tl > 6 ? (u32)(tl - 6) : 0u;        // top >> segshift < SEGS
    const u64 W = 1ull << ii.segshift;
    const int nseg = (int)(top >> ii.segshift) + 1;
    // how many entries each segment holds if every row's R entries are evenly spaced from its first to its last value
    constexpr double FIX = 65536.0;
    for (int p = tid; p < P; p += NT) {
        const u64 f = (u64)ends.value(p, 0) - (u64)base, l = (u64)ends.value(p, (u32)R - 1) - (u64)base;
        if (l < f || l > ii.range) continue;          // not a sorted row: the status says so elsewhere
        const u64 xf = f >> ii.wshift, xl = l >> ii.wshift;
        const u32 sf = (u32)(xf >> ii.segshift), sl = (u32)(xl >> ii.segshift);
        if (sf == sl) {
            atomicAdd(&seg_part[sf], (u64)((double)R * FIX));
        } else {
            const double rate = (double)R * FIX / (double)(xl - xf + 1);          // per unit of x
            atomicAdd(&seg_part[sf], (u64)(rate * (double)((((u64)sf + 1) << ii.segshift) - xf)));
            atomicAdd(&seg_part[sl], (u64)(rate * (double)(xl - ((u64)sl << ii.segshift) + 1)));
            if (sl > sf + 1) {
                const u64 whole = (u64)(rate * (double)W);
                atomicAdd(&seg_diff[sf + 1], whole);
                atomicAdd(&seg_diff[sl], 0ull - whole);
            }
        }
    }
    __syncthreads();
    if (tid < SEGS) {
        u64 cover = 0;
        for (int j = 0; j <= tid; ++j) cover += seg_diff[j];
        seg_est[tid] = tid < nseg ? seg_part[tid] + cover : 0;
    }
    __syncthreads();
    if (tid < SEGS) {
        u64 total = 0;
        for (int j = 0; j < nseg; ++j) total += seg_est[j];
        // an eighth of the bins is spread evenly, in case the rows are far from evenly spaced
        const u64 even = total / (8ull * (u64)nseg) + 1;
        const u64 total2 = total + even * (u64)nseg;
        u32 slope = 0;
        if (tid < nseg) {
            const u64 len = tid == nseg - 1 ? top - ((u64)tid << ii.segshift) + 1 : W;       // values of the segment in use
            const double share = (double)(seg_est[tid] + even) / (double)total2 * (double)(bins - 1);
            const double sl = share * 4294967296.0 / (double)len;
            slope = sl < 4294967295.0 ? (u32)sl : 0xffffffffu;
        }
        seg_step[tid] = W * (u64)slope;
        seg_slope[tid] = slope;
    }
    __syncthreads();
    if (tid < SEGS) {
        const u32 slope = seg_slope[tid];
        u64 G = 0;
        for (int j = 0; j < tid; ++j) G += seg_step[j];
        SegEntry e;
        e.G = G;
        e.slope = slope;
        e.pad_ = 0;
        segtab[b * (i64)SEGS + tid] = e;
        if (tid == nseg - 1) {
            ii.nb = (u32)((G + (top - ((u64)tid << ii.segshift)) * (u64)slope) >> 32) + 1u;
            info[b] = ii;
            if (status) status[b] = (int)ii.flags;
        }
    }
}

// zl_partition: one wave per row.  cross[row][k] = number of entries of the row
// that fall in fine bins below k, for k = 0..nb.
template <int NT, class CT>
__global__ __launch_bounds__(NT) void zl_partition_kernel(
    const i64* __restrict__ ts, i64 nrows, int P, int R,
    const InstInfo* __restrict__ info, const SegEntry* __restrict__ segtab, CT* __restrict__ cross, int stride,
    int* __restrict__ status)
{
    __shared__ SegEntry tabs[NT / WAVE][SEGS];         // each wave's copy of its instance's fine-bin map
    const int lane = threadIdx.x & (WAVE - 1);
    const i64 row_id = (i64)blockIdx.x * (NT / WAVE) + (threadIdx.x >> 6);
    if (row_id >= nrows) return;
    const i64 b = row_id / P;
    const InstInfo ii = info[b];
    SegEntry* tab = tabs[threadIdx.x >> 6];
    static_assert(SEGS == WAVE, "one entry per lane");
    tab[lane] = segtab[b * (i64)SEGS + lane];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");     // the wave's own stores, read by its other lanes below
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const i64* __restrict__ row = ts + row_id * (i64)R;
    CT* __restrict__ out = cross + row_id * (i64)stride;
    const u64 base = (u64)ii.base;

    int carry = -1;                        // bin of the element before lane 0's
    i64 carry_t = INT64_MIN;               // and its value
    bool bad = false;
    for (int i0 = 0; i0 < R; i0 += WAVE) {
        const int i = i0 + lane;
        int bin = -1;
        i64 t = INT64_MAX;
        if (i < R) { t = row[i]; bin = (int)fine_bin((u64)t - base, ii, tab); }
        int pb = __shfl_up(bin, 1, WAVE);
        i64 pt = __shfl_up(t, 1, WAVE);
        if (lane == 0) { pb = carry; pt = carry_t; }
        bad |= t < pt;                     // the only place the multi-window path checks every pair of neighbours
        if (i < R)
            for (int k = pb + 1; k <= bin; ++k) out[k] = (CT)i;
        carry = __shfl(bin, WAVE - 1, WAVE);
        carry_t = __shfl(t, WAVE - 1, WAVE);
    }
    if (__any(bad) && lane == 0 && status) atomicOr(status + b, (int)EBSP_STATUS_UNSORTED);
    const int last_bin = (int)fine_bin((u64)row[R - 1] - base, ii, tab);
    for (int k = last_bin + 1 + lane; k <= (int)ii.nb; k += WAVE) out[k] = (CT)R;
}

// The same with the column sums on the way: a workgroup takes PART_ROWS consecutive rows of
// one instance (one wave each), adds every crossing index it writes to an LDS array over
// the fine bins and stores that array as part[b][g][k] = sum of cross[p][k] over the rows p
// of group g.  zl_bincount then adds up P / PART_ROWS partial rows instead of P rows of
// cross.  For instances whose fine bins fit the LDS array (stride <= PART_MAX_STRIDE).
constexpr int PART_ROWS = 16;
constexpr int PART_MAX_STRIDE = 8200;
template <class CT>
__global__ __launch_bounds__(PART_ROWS * WAVE) void zl_partition_sum_kernel(
    const i64* __restrict__ ts, int P, int R, int groups,
    const InstInfo* __restrict__ info, const SegEntry* __restrict__ segtab, CT* __restrict__ cross, int stride,
    u32* __restrict__ part, int* __restrict__ status)
{
    constexpr int NT = PART_ROWS * WAVE;
    __shared__ SegEntry tab[SEGS];
    __shared__ u32 sums[PART_MAX_STRIDE];
    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    const i64 b = blockIdx.x / (u32)groups;
    const int g = (int)(blockIdx.x % (u32)groups);
    const int p = g * PART_ROWS + (tid >> 6);
    const InstInfo ii = info[b];
    if (tid < SEGS) tab[tid] = segtab[b * (i64)SEGS + tid];
    for (int k = tid; k <= (int)ii.nb; k += NT) sums[k] = 0;
    __syncthreads();
    if (p < P) {
        const i64 row_id = b * (i64)P + p;
        const i64* __restrict__ row = ts + row_id * (i64)R;
        CT* __restrict__ out = cross + row_id * (i64)stride;
        const u64 base = (u64)ii.base;
        int carry = -1;                        // bin of the element before lane 0's
        i64 carry_t = INT64_MIN;               // and its value
        bool bad = false;
        for (int i0 = 0; i0 < R; i0 += WAVE) {
            const int i = i0 + lane;
            int bin = -1;
            i64 t = INT64_MAX;
            if (i < R) { t = row[i]; bin = (int)fine_bin((u64)t - base, ii, tab); }
            int pb = __shfl_up(bin, 1, WAVE);
            i64 pt = __shfl_up(t, 1, WAVE);
            if (lane == 0) { pb = carry; pt = carry_t; }
            bad |= t < pt;                     // the only place the multi-window path checks every pair of neighbours
            if (i < R)
                for (int k = pb + 1; k <= bin; ++k) { out[k] = (CT)i; atomicAdd(&sums[k], (u32)i); }
            carry = __shfl(bin, WAVE - 1, WAVE);
            carry_t = __shfl(t, WAVE - 1, WAVE);
        }
        if (__any(bad) && lane == 0 && status) atomicOr(status + b, (int)EBSP_STATUS_UNSORTED);
        const int last_bin = (int)fine_bin((u64)row[R - 1] - base, ii, tab);
        for (int k = last_bin + 1 + lane; k <= (int)ii.nb; k += WAVE) { out[k] = (CT)R; atomicAdd(&sums[k], (u32)R); }
    }
    __syncthreads();
    u32* __restrict__ mine = part + (b * (i64)groups + g) * stride;
    for (int k = tid; k <= (int)ii.nb; k += NT) mine[k] = sums[k];
}

// zl_partition for predicted rows: the same crossing indices from arithmetic.  Row p
// holds first + i * step (i < R, relative to the instance's base); the entries in
// fine bins below k are those below the first value of bin k.  One thread per bin
// (consecutive threads write consecutive indices of a row), looping over the rows.
constexpr int PRED_ROWS_PER_BLOCK = 64;
template <class CT>
__global__ __launch_bounds__(256) void zl_partition_pred_kernel(
    const i64* __restrict__ le, const i64* __restrict__ iv, int P, int R,
    const InstInfo* __restrict__ info, const SegEntry* __restrict__ segtab, CT* __restrict__ cross, int stride,
    u32* __restrict__ part)
{
    const u32 kblocks = (u32)(stride + 255) / 256;
    const i64 b = blockIdx.x / kblocks;
    const int k = (int)(blockIdx.x % kblocks) * 256 + (int)threadIdx.x;
    const int p_begin = (int)blockIdx.y * PRED_ROWS_PER_BLOCK;           // a slice of the rows per workgroup
    const int p_end = p_begin + PRED_ROWS_PER_BLOCK < P ? p_begin + PRED_ROWS_PER_BLOCK : P;
    const InstInfo ii = info[b];
    if (k > (int)ii.nb) return;
    const bool broken = (ii.flags & EBSP_STATUS_UNSORTED) != 0;      // a negative interval: indices stay zero
    const u64 edge = k >= (int)ii.nb ? U64_MAX : fine_bin_start((u32)k, ii, segtab + b * (i64)SEGS);   // bin nb: everything lies below
    const i64* __restrict__ lep = le + b * (i64)P;
    const i64* __restrict__ ivp = iv + b * (i64)P;
    CT* __restrict__ out = cross + (b * (i64)P) * stride + k;
    const bool narrow_values = (ii.range >> 32) == 0;
    u32 sum = 0;
    for (int p = p_begin; p < p_end; ++p) {
        const u64 step = (u64)ivp[p];
        const u64 first = (u64)lep[p] + step - (u64)ii.base;
        u64 below;                                                   // entries with first + i * step < edge
        if (broken) below = 0;
        else if (edge == U64_MAX) below = (u64)R;
        else if (edge <= first) below = 0;
        else if (step == 0) below = (u64)R;
        else if (narrow_values && (step >> 32) == 0) below = (u64)(((u32)(edge - first) - 1u) / (u32)step) + 1u;
        else below = (edge - first - 1) / step + 1;
        const u32 c = (u32)(below < (u64)R ? below : (u64)R);
        out[(i64)p * stride] = (CT)c;
        sum += c;
    }
    part[(b * (i64)gridDim.y + blockIdx.y) * stride + k] = sum;      // this slice's share of the column sum
}

// zl_bincount: below[b][k] = number of keys of instance b under fine bin k, k = 0..nb:
// the column sums of cross.  Exact, so that zl_plan can fill windows to the brim.
// A thread sums four neighbouring columns (one 8- or 16-byte load per row; `stride`
// is a multiple of 8), the four waves of a workgroup take every fourth row each.
template <class CT>
__global__ __launch_bounds__(256) void zl_bincount_kernel(
    const CT* __restrict__ cross, int P, int R, int stride,
    const InstInfo* __restrict__ info, u32* __restrict__ below)
{
    struct alignas(4 * sizeof(CT)) Four { CT v[4]; };
    __shared__ u32 part[4][256];
    const int tid = threadIdx.x, kl = tid & 63, pg = tid >> 6;
    const u32 kblocks = (u32)(stride + 255) / 256;
    const i64 b = blockIdx.x / kblocks;
    const int k = (int)(blockIdx.x % kblocks) * 256 + 4 * kl;          // k .. k + 3, all below stride or none
    const u32 nb = info[b].nb;
    u32 s0 = 0, s1 = 0, s2 = 0, s3 = 0;
    if (k <= (int)nb) {
        const CT* col = cross + (b * (i64)P) * stride + k;
#pragma unroll 8
        for (int p = pg; p < P; p += 4) {
            const Four c = *(const Four*)(col + (i64)p * stride);
            s0 += c.v[0] < (u32)R ? (u32)c.v[0] : (u32)R;
            s1 += c.v[1] < (u32)R ? (u32)c.v[1] : (u32)R;
            s2 += c.v[2] < (u32)R ? (u32)c.v[2] : (u32)R;
            s3 += c.v[3] < (u32)R ? (u32)c.v[3] : (u32)R;
        }
    }
    part[0][tid] = s0; part[1][tid] = s1; part[2][tid] = s2; part[3][tid] = s3;
    __syncthreads();
    if (pg == 0)
        for (int c = 0; c < 4; ++c)
            if (k + c <= (int)nb)
                below[b * (i64)stride + k + c] = part[c][kl] + part[c][64 + kl] + part[c][128 + kl] + part[c][192 + kl];
}

// zl_plan: windows of an instance.  below[] holds the exact number of keys under
// every fine bin, so the windows are packed greedily: a window takes fine bins while
// its entries stay within `fill` (a bin larger than that becomes a window of its own,
// which the window kernel leaves to the general search).  The packing is a sequential
// walk over the bins by one wave (64 bins at a time, one ballot per window), fed from
// LDS in slices the workgroup loads together; the per-window values follow in parallel.  Per window: its first fine bin
// (winstart), its first and last value and the constants of the linear bucket map
// over that span (winval).
struct WinVal {
    u64 A, Elast;
    u64 inv52;     // floor(2^52 / scale)
    u32 scale;     // linear_scale(Elast - A, buckets), when the span fits 32 bits
    u32 pad_;
};

template <int NT, int PLAN_SLICE>       // PLAN_SLICE: fine bins held in LDS at a time
__global__ __launch_bounds__(NT) void zl_plan_kernel(
    InstInfo* __restrict__ info, const SegEntry* __restrict__ segtab, const u32* __restrict__ below, int stride,
    u32* __restrict__ winstart, WinVal* __restrict__ winval, int max_win, u32 fill, u32 buckets)
{
    __shared__ u32 ends[PLAN_SLICE + 1];   // ends[i + 1] = keys under bin k0 + i + 1 = where bin k0 + i ends
    __shared__ u32 found_all;
    __shared__ SegEntry tab[SEGS];         // the instance's fine-bin map
    __shared__ u16 hop[2][PLAN_SLICE + 1];
    const int tid = threadIdx.x;
    const i64 b = blockIdx.x;
    const u32* bel = below + b * (i64)stride;
    u32* ws = winstart + b * (i64)(max_win + 1);
    WinVal* wv = winval + b * (i64)max_win;
    const InstInfo ii = info[b];
    const int nb = (int)ii.nb;
    if (tid == 0) found_all = 0;
    if (nb <= PLAN_SLICE) {
        // All bins fit in LDS.  jump[k] = the bin that opens the next window if one opens at bin k
        // (nb: none); the windows open at 0, jump[0], jump[jump[0]], ...  Thread r finds the r-th
        // of them by squaring the jump table: level l applies jump^(2^l) to the ranks with bit l set.
        static_assert(PLAN_SLICE % NT == 0, "whole ranks per thread");
        constexpr int RANKS = PLAN_SLICE / NT;          // ranks per thread: every window holds at least one bin
        u16* jump = hop[0];
        u16* other = hop[1];
        for (int i = tid; i <= nb; i += NT) ends[i] = bel[i];
        __syncthreads();
        for (int k = tid; k <= nb; k += NT) {
            int lo = k + 1, hi = nb;                      // first bin j > k whose end lies more than `fill` past the start of bin k
            if (k < nb) {
                const u32 limit = ends[k] + fill;         // no overflow: fill and the key count are both below 2^31
                while (lo < hi) { const int m = (lo + hi) >> 1; if (ends[m + 1] > limit) hi = m; else lo = m + 1; }
            } else lo = nb;
            jump[k] = (u16)lo;
        }
        u32 pos[RANKS];
#pragma unroll
        for (int q = 0; q < RANKS; ++q) pos[q] = 0;
        const u32 top_rank = (u32)nb < (u32)max_win ? (u32)nb : (u32)max_win;
        for (int level = 0; (1u << level) <= top_rank; ++level) {
            __syncthreads();
#pragma unroll
            for (int q = 0; q < RANKS; ++q)
                if (((u32)(q * NT + tid) >> level) & 1u) pos[q] = jump[pos[q]];
            for (int k = tid; k <= nb; k += NT) other[k] = jump[jump[k]];
            u16* t = jump; jump = other; other = t;
        }
#pragma unroll
        for (int q = 0; q < RANKS; ++q) {
            const u32 r = (u32)(q * NT + tid);
            if (pos[q] < (u32)nb && r < (u32)max_win) {
                ws[r] = pos[q];
                atomicMax(&found_all, r + 1);
            }
        }
        __syncthreads();
        if (tid == 0) { ws[found_all] = (u32)nb; info[b].nwin = found_all; }
    } else {
    // wave 0 walks the bins, 64 at a time: one step per window, not per bin
    u32 found = 0, first_key = 0;          // windows so far, keys under the open window's first bin
    for (int k0 = 0; k0 < nb; k0 += PLAN_SLICE) {
        const int cnt = nb - k0 < PLAN_SLICE ? nb - k0 : PLAN_SLICE;
        __syncthreads();
#pragma unroll 4
        for (int i = tid; i <= cnt; i += NT) ends[i] = bel[k0 + i];
        __syncthreads();
        if (tid < WAVE) {
            for (int i0 = 0; i0 < cnt; i0 += WAVE) {
                const int i = i0 + tid;
                const bool valid = i < cnt;
                const u32 e = valid ? ends[i + 1] : 0u;
                const u32 before = valid ? ends[i] : 0u;            // where the bin before this one ends
                int from = 0;
                for (;;) {
                    const bool opens = valid && tid >= from && (k0 + i == 0 || e - first_key > fill);
                    const unsigned long long m = __ballot(opens);
                    if (!m) break;
                    const int at = __builtin_amdgcn_readfirstlane(__ffsll((long long)m) - 1);   // bin k0 + i0 + at opens a window
                    if (tid == at && found < (u32)max_win) ws[found] = (u32)(k0 + i);
                    ++found;
                    first_key = (u32)__builtin_amdgcn_readlane((int)before, at);
                    from = at + 1;
                }
            }
        }
    }
    if (tid == 0) {
        // more starts than max_win cannot come from sorted rows; the last window then runs to the end
        const u32 nwin = found < (u32)max_win ? found : (u32)max_win;
        ws[nwin] = (u32)nb;
        info[b].nwin = nwin;
        found_all = nwin;
    }
    }
    if (tid < SEGS) tab[tid] = segtab[b * (i64)SEGS + tid];
    __threadfence_block();
    __syncthreads();
    const u32 nwin = found_all;
    for (u32 j = tid; j < nwin; j += NT) {
        const u64 first = fine_bin_start(ws[j], ii, tab);
        const u64 last = j + 1 < nwin ? fine_bin_start(ws[j + 1], ii, tab) - 1 : ii.range;
        const u64 span = last - first;
        const u32 scale = linear_scale(span <= 0xffffffffull ? span : 0xffffffffull, buckets);
        WinVal v;
        v.A = first;
        v.Elast = last;
        v.scale = scale;
        v.inv52 = (1ull << 52) / scale;
        v.pad_ = 0;
        wv[j] = v;
    }
}

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

// The fast search of one window (see zl_window_kernel); lo/hi hold the index
// ranges of the thread's first ROWS_PER_THREAD<NT> rows.
template <int NT, int ITEMS, class CT, bool PRED>
__device__ __forceinline__ void window_search(const Smem& sm, const Rows& rw, const WinVal& wv, const InstInfo& ii, bool hot,
                                              const u32 (&lo)[ROWS_PER_THREAD<NT>], const u32 (&hi)[ROWS_PER_THREAD<NT>],
                                              Partial* __restrict__ out)
{
    using H = HotCfg<NT, ITEMS>;
    {
        u64* bsum = sm.recs + H::BSUM_AT;
        bsum[threadIdx.x] = 0; bsum[threadIdx.x + NT] = 0;
    }
    Partial r;
    r.wait = U64_MAX;
    r.brel = 0;
    if (wv.Elast >= wv.A) {
        bool defer = !hot;
        if (!defer) {
            u32 key[ITEMS], dl[ITEMS];
            u64 w0 = 0;
            const int total = zl_delta_rows<NT, ITEMS, CT, PRED>(sm, rw, wv.A, H::CAP, lo, hi, key, dl, w0);
            defer = total > H::CAP;
            if (!defer && total > 0) {
                u32 bkey;
                if (zl_bucket_finish<NT, ITEMS, true>(sm, key, dl,
                                                      linear_map((u32)(wv.Elast - wv.A), H::NB, wv.scale ? wv.scale : 1u,
                                                                 wv.inv52),
                                                      total, wv.A, ii.thr, (u32)rw.P, w0, r.wait, bkey))
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
    const bool hot = !(ii.range >> 32) && (u64)P * (u64)R < HOT_MAX_ENTRIES;
    Rows rw;
    rw.inst = PRED ? nullptr : ts + b * (i64)P * R;
    rw.le = nullptr; rw.iv = nullptr;
    rw.par = PRED ? rowpar + b * (i64)P : nullptr;
    rw.P = P; rw.R = R; rw.base = (u64)ii.base;
    rw.cr = (const void*)(cross + (b * (i64)P) * stride);
    rw.narrow = sizeof(CT) == 2;
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
__global__ __launch_bounds__(NT, 4) void zl_window_kernel(
    const i64* __restrict__ ts, const uint2* __restrict__ rowpar, i64 B, int P, int R,
    const InstInfo* __restrict__ info, const CT* __restrict__ cross, int stride,
    const u32* __restrict__ winstart, const WinVal* __restrict__ winval, int max_win, u32 groups, u32 groups_inv,
    Partial* __restrict__ partial)
{
    using H = HotCfg<NT, ITEMS, false>;       // windows use the linear bucket map: no coarse table
    __shared__ __align__(16) unsigned char smem[H::BYTES];
    const Smem sm = carve_hot<NT, ITEMS>(smem);
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

// ---------------------------------------------------------------------------
// The paper's formal objective (Section III): d_Z = max(Z) - min(Z).  For a barrier
// c the tightest Z holds every worker's latest timestamp <= c, so
// d(c) = c - min_p last_p(c); the search returns the first minimum over the
// timestamps c >= max_p t[p][0] (Algorithm 2 evaluates exactly these states of Z).
//
// One value interval [a, el] of the rows in `rw` (all of an instance, or one window
// of the multi-window path) is handled by one workgroup: the entries are gathered as
// (key = value - a, next = the same worker's next value - a, or NEVER) plus, for the
// first entry of a row inside the interval, gone = a - the worker's last value
// before the interval (NEVER if the worker has none: it has not finished an
// iteration yet), and sorted by key (zl_sort).  At sorted position k:
//   * a worker whose first entry in the interval lies at a position > k (or that has
//     no entry in it) still stands at its value before the interval: the largest
//     `gone` over those workers, G(k), is a suffix maximum, and d = key_k + G(k);
//   * if there is no such worker, min(Z) is the first entry j whose successor has
//     not arrived yet (next_j > key_k): with M(j) the prefix maximum of next,
//     j = #{ j' : M(j') <= key_k } (M is monotone: a binary search), d = key_k - key_j.
// Entries equal to key_k at later positions are treated as not yet arrived; that can
// only raise d at position k, and the last position of the run of equal keys sees
// them all, so the minimum over all positions is the minimum over the timestamps.
// Needs a value spread below 2^32 - 1 (keys and the NEVER mark share 32 bits).
constexpr u32 NEVER = 0xffffffffu;

template <class T, int NT, class Op>
__device__ __forceinline__ T block_excl_scan_op(T v, T* red, Op op)      // `red` holds NT/64 T's
{
    constexpr int NW = NT / WAVE;
    constexpr T id = Op::template identity<T>();
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x >> 6;
    const T inc = wave_scan(v, op);
    if (lane == WAVE - 1) red[wave] = inc;
    T before = dpp_take<DPP_WAVE_SHR1, 0xf>(id, inc);       // exclusive inside the wave
    if (lane == 0) before = id;
    __syncthreads();
    T base = id;
#pragma unroll 4
    for (int w = 0; w < NW; ++w)
        if (w < wave) base = op(base, red[w]);
    __syncthreads();
    return op(base, before);
}

// Gather for the range objective; returns the number of entries (nothing useful is
// stored if it exceeds `cap`).  absent = the largest `gone` over the workers without
// an entry in the interval (this thread's share).
template <int NT>
__device__ __forceinline__ int zl_range_gather(const Smem& sm, const Rows& rw, u64 a, u64 el, bool lx, bool rx,
                                               int cap, u32& absent, int& bad)
{
    const int tid = threadIdx.x;
    u32* rowoff = sm.cnt;
    u32* rowlo = sm.cnt + NT;
    int total = 0;
    for (int p0 = 0; p0 < rw.P; p0 += NT) {
        const int p = p0 + tid;
        u32 lo = 0, hi = 0;
        if (p < rw.P) {
            sub_range(rw, p, a, el, lx, rx, lo, hi);
            if (lo == hi) {
                const u32 gone = lo > 0 ? (u32)(a - rw.rel(p, lo - 1)) : NEVER;
                absent = gone > absent ? gone : absent;
            }
        }
        u32 chunk;
        const u32 off = block_excl_scan<u32, NT>(hi - lo, (u32*)sm.red, chunk);
        rowoff[tid] = off;
        rowlo[tid] = lo;
        __syncthreads();
        const int room = cap - total;
        const int take = (int)chunk < room ? (int)chunk : room;
        const int nrows = (rw.P - p0) < NT ? (rw.P - p0) : NT;
        for (int e = tid; e < take; e += NT) {
            int l = 0, h = nrows;                 // the last row r with rowoff[r] <= e
            while (h - l > 1) {
                const int m = (l + h) >> 1;
                if (rowoff[m] <= (u32)e) l = m; else h = m;
            }
            const u32 i = rowlo[l] + ((u32)e - rowoff[l]);
            const i64* src = rw.inst + (size_t)(p0 + l) * rw.R + i;
            const i64 cur = src[0];
            const u64 rel = (u64)cur - rw.base;
            u32 next = NEVER, gone = 0;
            if (i + 1 < (u32)rw.R) {
                const i64 nxt = src[1];
                bad |= (nxt < cur);
                next = (u32)((u64)nxt - rw.base - a);
            }
            if (i == rowlo[l]) {                  // the row's first entry inside the interval
                gone = NEVER;
                if (i > 0) {
                    const i64 prv = src[-1];
                    bad |= (cur < prv);
                    gone = (u32)(a - ((u64)prv - rw.base));
                }
            }
            const int slot = phys(total + e);
            sm.recs[slot] = (u64)(u32)(rel - a) | ((u64)next << 32);
            sm.dhi[slot] = gone;
        }
        total += (int)chunk;
        __syncthreads();
    }
    return total;
}

// The search over the sorted entries [0, total); thread t owns positions
// [t*items, (t+1)*items).  Returns the first minimum (d, key); d == U64_MAX: none.
template <int NT>
__device__ __forceinline__ void zl_range_scan_argmin(const Smem& sm, int items, int total, u64 a, u64 thr,
                                                     u32 absent_all, u64& best_d, u32& best_key)
{
    u64* recs = sm.recs;
    u32* gone = sm.dhi;
    u32* mirror = sm.cnt;                        // NT words
    const int tid = threadIdx.x;
    const int q0 = tid * items < total ? tid * items : total;
    const int qe = q0 + items < total ? q0 + items : total;
    // M: prefix maximum of `next`, written over `next`
    u32 mine = 0;
    for (int q = q0; q < qe; ++q) { const u32 nx = (u32)(recs[phys(q)] >> 32); mine = nx > mine ? nx : mine; }
    u32 run = block_excl_scan_op<u32, NT>(mine, (u32*)sm.red, OpMax());
    for (int q = q0; q < qe; ++q) {
        const u64 r = recs[phys(q)];
        const u32 nx = (u32)(r >> 32);
        run = nx > run ? nx : run;
        recs[phys(q)] = (u64)(u32)r | ((u64)run << 32);
    }
    // G: largest `gone` over the positions behind the thread's own (threads in mirrored order)
    u32 far = 0;
    for (int q = q0; q < qe; ++q) { const u32 g = gone[phys(q)]; far = g > far ? g : far; }
    mirror[NT - 1 - tid] = far;
    __syncthreads();
    const u32 mv = mirror[tid];
    __syncthreads();
    const u32 behind_m = block_excl_scan_op<u32, NT>(mv, (u32*)sm.red, OpMax());   // for thread NT-1-tid
    mirror[NT - 1 - tid] = behind_m;
    __syncthreads();                              // also: every M is in place
    u32 G = mirror[tid];
    G = absent_all > G ? absent_all : G;

    u64 bd = U64_MAX;
    u32 bq = 0xffffffffu, bk = 0;
    for (int q = qe - 1; q >= q0; --q) {          // right to left: G covers the positions behind q
        const u32 key = (u32)recs[phys(q)];
        if (a + key >= thr && G != NEVER) {
            u64 d;
            bool ok = true;
            if (G > 0) {
                d = (u64)key + G;
            } else {
                int l = 0, h = total;             // number of positions j with M(j) <= key
                while (l < h) {
                    const int m = (l + h) >> 1;
                    if ((u32)(recs[phys(m)] >> 32) <= key) l = m + 1; else h = m;
                }
                ok = l < total;
                d = ok ? (u64)(key - (u32)recs[phys(l)]) : 0;
            }
            if (ok && (d < bd || (d == bd && (u32)q < bq))) { bd = d; bq = (u32)q; bk = key; }
        }
        const u32 g = gone[phys(q)];
        G = g > G ? g : G;
    }
    // block arg-min over (d, position): smaller d, then earlier position
    u64 pk = ((u64)bq << 32) | bk;
    wave_argmin(bd, pk);
    constexpr int NW = NT / WAVE;
    const int lane = tid & (WAVE - 1), wave = tid >> 6;
    u64* red = sm.red;
    __syncthreads();
    if (lane == WAVE - 1) { red[wave] = bd; red[NW + wave] = pk; }
    __syncthreads();
    bd = red[0]; pk = red[NW];
#pragma unroll 4
    for (int w = 1; w < NW; ++w) {
        const u64 od = red[w], ok = red[NW + w];
        if (od < bd || (od == bd && ok < pk)) { bd = od; pk = ok; }
    }
    __syncthreads();
    best_d = bd;
    best_key = (u32)pk;
}

// One interval [A, Elast] (less than 2^32 - 1 wide): gather, sort, search.  An interval
// with more than CAP_WIDE entries is walked in pieces that do fit, cut by bisection on
// the value (every piece is searched on its own: what a piece needs from outside it
// are the neighbouring entries of its rows, which the gather reads); a single value
// that alone occurs more than CAP_WIDE times is one candidate and is evaluated
// directly from the rows.  (bd, bb) is updated with the first minimum found.
template <int NT, int ITEMS>
__device__ __forceinline__ void zl_range_window(const Smem& sm, const Rows& rw, u64 thr, u64 A, u64 Elast,
                                                u64& bd, u64& bb, int& bad)
{
    using C = WinCfg<NT, ITEMS>;
    constexpr int CAPW = C::CAP_WIDE;
    u64 a = A;
    bool lx = true;
    for (;;) {
        u64 el = Elast;
        bool rx = true;
        u32 absent = 0;
        int total = zl_range_gather<NT>(sm, rw, a, el, lx, rx, CAPW, absent, bad);
        bool single = false;
        if (total > CAPW) {
            if (count_interval<NT>(sm, rw, a, a, lx) > (u32)CAPW) {
                single = true;                     // the value `a` alone overflows a piece
                el = a;
            } else {
                u64 l = a, h = el;                 // count(a, l) <= CAPW < count(a, h)
                while (h - l > 1) {
                    const u64 m = l + ((h - l) >> 1);
                    if (count_interval<NT>(sm, rw, a, m, lx) <= (u32)CAPW) l = m; else h = m;
                }
                el = l;
                absent = 0;
                total = zl_range_gather<NT>(sm, rw, a, el, lx, false, CAPW, absent, bad);
            }
            rx = false;
        }
        if (single) {
            // candidate c = a: every row stops at its last entry <= a
            u64 far = 0;
            int missing = 0;
            for (int p = threadIdx.x; p < rw.P; p += NT) {
                u32 lo, hi;
                sub_range(rw, p, a, a, lx, false, lo, hi);
                if (hi > 0) { const u64 g = a - rw.rel(p, hi - 1); far = g > far ? g : far; } else missing = 1;
            }
            const u64 d = block_reduce<u64, NT>(far, sm.red, OpMax());
            missing = __syncthreads_or(missing);
            if (!missing && a >= thr && (d < bd || (d == bd && a < bb))) { bd = d; bb = a; }
        } else {
            const u32 absent_all = block_reduce<u32, NT>(absent, (u32*)sm.red, OpMax());   // also orders the record writes
            if (total > 0) {
                const int items = (total + NT - 1) / NT;
                fill_sentinels<NT>(sm.recs, total, items);
                __syncthreads();
                zl_sort<NT, ITEMS, true>(sm, items, bit_length(el - a));
                u64 d;
                u32 key;
                zl_range_scan_argmin<NT>(sm, items, total, a, thr, absent_all, d, key);
                if (d != U64_MAX && (d < bd || (d == bd && a + key < bb))) { bd = d; bb = a + key; }
            }
        }
        if (rx) break;
        // continue at the smallest entry above el, if any
        u64 nxt = U64_MAX;
        int have = 0;
        for (int p = threadIdx.x; p < rw.P; p += NT) {
            u32 lo, hi;
            rw.range(p, lo, hi);
            const u32 i = row_lower_bound(rw, p, lo, hi, el + 1);
            if (i < hi) { const u64 v = rw.rel(p, i); nxt = v < nxt ? v : nxt; have = 1; }
        }
        nxt = block_reduce<u64, NT>(nxt, sm.red, OpMin());
        have = __syncthreads_or(have);
        if (!have || nxt > Elast || nxt <= el) break;
        a = nxt;
        lx = false;
    }
}

// ---------------------------------------------------------------------------
// The fast form of the range search for one window of the multi-window path:
// value buckets instead of a sort, as for the summed wait.  With next(x) = the same
// worker's next value and gone(x) = how far the worker's previous value lies
// before the window (for a row's first entry in it; 0 otherwise),
//   min(Z) at time c  =  - max{ gone(x) : x > c }              if that is positive
//                        (some worker still stands before the window), else
//                     =  min{ x <= c : next(x) > c }.
// Per bucket b: reach(b) = max next, far(b) = max gone, both by LDS atomics while the
// entries are gathered.  M = prefix maximum of reach, F = suffix maximum of far.  The
// entry that is min(Z) at time c lies in the first bucket with M > c, so for every c
// of bucket b: lo(first bucket with M > lo(b)) <= min(Z) <= hi(first bucket with M >
// hi(b)) (or -F on either side while F > 0): an upper bound of d for some candidate of
// the bucket and a lower bound for all of them.  Buckets whose lower bound exceeds the
// smallest upper bound are dropped.  For the candidates that remain, and for the
// entries of the buckets that can hold their min(Z) (buckets where M rises, between
// the bounds of the remaining candidates), key, next and gone are read again through
// the source words and d is evaluated exactly from that short list.
// Returns false if the window has to be left to the sort-based search (too many
// entries for the list to fit behind them, or too many listed).


template <int NT, int ITEMS, class CT>
__device__ __forceinline__ bool zl_range_bucket_search(const Smem& sm, const Rows& rw, const WinVal& wv, u64 thr,
                                                       const u32 (&lo)[ROWS_PER_THREAD<NT>],
                                                       const u32 (&hi)[ROWS_PER_THREAD<NT>],
                                                       u64& best_d, u32& best_key)
{
    using H = HotCfg<NT, ITEMS, false>;
    constexpr int NB = H::NB;
    constexpr int NW = NT / WAVE;
    static_assert(NB == 2 * NT, "two buckets per thread");
    constexpr int RANGE_LIST_CAP = 2 * NT;                  // entries of the short list (four words each, behind the source words)
    const int tid = threadIdx.x;
    u64* recs = sm.recs;
    u32* reach = (u32*)(sm.recs + H::BSUM_AT);              // NB words, later M
    u32* far = reach + NB;                                  // NB words, later F (exclusive)
    u32* flag = sm.cnt;                                     // NB words: entry counts, later what a bucket is kept for
    u32* misc = (u32*)(sm.red + H::RED_WORDS - 3);          // listed holders, lowest and highest kept value, absent rows, listed others
    reach[tid] = 0; reach[tid + NT] = 0;
    far[tid] = 0; far[tid + NT] = 0;
    flag[tid] = 0; flag[tid + NT] = 0;
    if (tid == 0) { misc[0] = 0; misc[1] = 0xffffffffu; misc[2] = 0; misc[3] = 0; misc[4] = 0; }
    const char* bytes = (const char*)rw.inst;
    const u64 a = wv.A;
    const u32 start = (u32)(rw.base + a);                   // low word of the window's first value
    u64 unused = 0;
    u32 absent = 0;
    const int total = zl_place_rows<NT, CT, false, true>(sm, rw, start, H::CAP, lo, hi, unused, absent);
    best_d = U64_MAX;
    best_key = 0;
    if (total > H::CAP - 2 * RANGE_LIST_CAP) return false;
    if (total == 0) return true;
    const LinearMap bucket = linear_map((u32)(wv.Elast - a), NB, wv.scale ? wv.scale : 1u, wv.inv52);
    auto read_entry = [&](u64 src, u32& key, u32& next, u32& gone) {     // an entry through its source word
        const u32 at = (u32)src;
        const bool inner = (src & FIRST_OF_SEGMENT) && !(src & FIRST_OF_ROW);   // has a predecessor before the window
        const bool last = (src & LAST_OF_ROW) != 0;
        const u32 cur = *(const u32*)(bytes + (at << 3));
        const u32 nxt = *(const u32*)(bytes + ((at + (last ? 0u : 1u)) << 3));
        const u32 prv = *(const u32*)(bytes + ((at - (inner ? 1u : 0u)) << 3));
        key = cur - start;
        next = last ? NEVER : nxt - start;
        gone = inner ? start - prv : 0u;
    };
    // sweep 2: reach, far and the entry count of every bucket; the keys stay in registers
    u32 key[ITEMS];
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const int q = j * NT + tid;
        key[j] = 0;
        if (j * NT < total) {
            u32 next, gone;
            read_entry(q < total ? recs[q] : (FIRST_OF_ROW | LAST_OF_ROW), key[j], next, gone);
            if (q < total) {
                const u32 b = bucket(key[j]);
                atomicAdd(&flag[b], 1u);
                atomicMax(&reach[b], next);
                if (gone) atomicMax(&far[b], gone);
            }
        }
    }
    if (absent) atomicMax(&misc[3], absent);
    __syncthreads();
    const u32 absent_all = misc[3];
    const u32 c0 = flag[2 * tid], c1 = flag[2 * tid + 1];
    const u32 r0 = reach[2 * tid], r1 = reach[2 * tid + 1];
    const u32 g0 = far[2 * tid], g1 = far[2 * tid + 1];
    // M: prefix maximum of reach (inclusive), F: maximum of far over the buckets behind (and the absent rows)
    const u32 m_before = block_excl_scan_op<u32, NT>(r0 > r1 ? r0 : r1, (u32*)sm.red, OpMax());
    const u32 M0 = m_before > r0 ? m_before : r0, M1 = M0 > r1 ? M0 : r1;
    u32* mirror = (u32*)(recs + ((total + 1) & ~1));        // NT words behind the source words
    mirror[NT - 1 - tid] = g0 > g1 ? g0 : g1;
    __syncthreads();
    const u32 mv = mirror[tid];
    __syncthreads();
    const u32 behind_m = block_excl_scan_op<u32, NT>(mv, (u32*)sm.red, OpMax());
    mirror[NT - 1 - tid] = behind_m;
    __syncthreads();
    u32 F1 = mirror[tid];                                   // buckets behind 2*tid + 1
    F1 = absent_all > F1 ? absent_all : F1;
    const u32 F0 = g1 > F1 ? g1 : F1;                       // buckets behind 2*tid
    reach[2 * tid] = M0; reach[2 * tid + 1] = M1;
    far[2 * tid] = g0 > F0 ? g0 : F0;                       // from here on: the bucket itself included
    far[2 * tid + 1] = g1 > F1 ? g1 : F1;
    __syncthreads();
    // bounds of d over each bucket
    const u64 need = thr > a ? thr - a : 0;                 // keys >= need are admissible
    u32 lo0, hi0, lo1, hi1;
    bucket.bounds_pair(2 * tid, lo0, hi0, lo1, hi1);
    auto first_above = [&](u32 v) {                          // first bucket with M > v (NB if none)
        int l = 0, h = NB;
        while (l < h) { const int m = (l + h) >> 1; if (reach[m] > v) h = m; else l = m + 1; }
        return l;
    };
    auto bounds_of = [&](u32 k, u32 c, u32 g, u32 F, u32 lok, u32 hik, i64& ub, i64& lb) {
        ub = INT64_MAX; lb = INT64_MAX;
        if (!c) return;
        const u32 Fin = g > F ? g : F;                       // workers that may still stand before the window
        i64 zlow, zhigh;                                     // min(Z) over the bucket lies in [zlow, zhigh]
        if (Fin) zlow = -(i64)Fin;
        else {
            u32 jl = (u32)first_above(lok);
            jl = jl < k ? jl : k;
            u32 l2, h2;
            bucket.bounds(jl, l2, h2);
            zlow = (i64)l2;
        }
        if (F) zhigh = -(i64)F;
        else {
            const u32 jh = (u32)first_above(hik);
            u32 l2, h2 = hik;
            if (jh < k) bucket.bounds(jh, l2, h2);
            zhigh = (i64)(h2 < hik ? h2 : hik);
        }
        lb = (i64)lok - zhigh;
        if ((u64)lok >= need) ub = (i64)hik - zlow;
    };
    i64 ub0, lb0, ub1, lb1;
    bounds_of(2 * tid, c0, g0, F0, lo0, hi0, ub0, lb0);
    bounds_of(2 * tid + 1, c1, g1, F1, lo1, hi1, ub1, lb1);
    const i64 ubmin = block_reduce<i64, NT>(ub0 < ub1 ? ub0 : ub1, (i64*)sm.red, OpMin());
    const bool live0 = c0 && (u64)hi0 >= need && lb0 <= ubmin;
    const bool live1 = c1 && (u64)hi1 >= need && lb1 <= ubmin;
    if (live0 || live1) {
        atomicMin(&misc[1], live0 ? lo0 : lo1);
        atomicMax(&misc[2], live1 ? hi1 : hi0);
    }
    __syncthreads();
    const u32 clo = misc[1], chi = misc[2];                 // all remaining candidates lie in [clo, chi]
    // buckets where M rises hold the entries that are min(Z) at some time: those between clo and chi
    const bool holds0 = r0 > m_before && M0 > clo && m_before <= chi;
    const bool holds1 = r1 > M0 && M1 > clo && M0 <= chi;
    flag[2 * tid] = (live0 ? 1u : 0u) | (holds0 ? 2u : 0u);
    flag[2 * tid + 1] = (live1 ? 1u : 0u) | (holds1 ? 2u : 0u);
    __syncthreads();
    // the short list: slot and purpose first, then the entries themselves.  Entries of the
    // buckets that can hold min(Z) fill it from the front, mere candidates from the back.
    u32* lslot = mirror;                                    // RANGE_LIST_CAP words each
    u32* lkey = lslot + RANGE_LIST_CAP;
    u32* lnext = lkey + RANGE_LIST_CAP;
    u32* lgone = lnext + RANGE_LIST_CAP;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const int q = j * NT + tid;
        if (q < total) {
            const u32 f = flag[bucket(key[j])];
            if (f & 2u) {
                const u32 at = atomicAdd(&misc[0], 1u);
                if (at < (u32)RANGE_LIST_CAP) lslot[at] = (u32)q | (f << 16);
            } else if (f) {
                const u32 at = atomicAdd(&misc[4], 1u);
                if (at < (u32)RANGE_LIST_CAP) lslot[RANGE_LIST_CAP - 1 - at] = (u32)q | (f << 16);
            }
        }
    }
    __syncthreads();
    const int holders = (int)misc[0], others = (int)misc[4];
    if (holders + others > RANGE_LIST_CAP) return false;
    const int back = RANGE_LIST_CAP - others;               // the list is [0, holders) and [back, RANGE_LIST_CAP)
    for (int i = tid; i < holders + others; i += NT) {
        const int e = i < holders ? i : back + (i - holders);
        read_entry(recs[lslot[e] & 0xffffu], lkey[e], lnext[e], lgone[e]);
    }
    __syncthreads();
    u64 bd = U64_MAX;
    u32 bk = 0xffffffffu;
    for (int i = tid; i < holders + others; i += NT) {
        const int me = i < holders ? i : back + (i - holders);
        if (!(lslot[me] & 0x10000u)) continue;              // not a candidate, only a possible min(Z)
        const u32 c = lkey[me];
        if ((u64)c < need) continue;
        const u32 b = bucket(c);
        u32 out = 0;                                         // how far back the workers stand whose first entry lies behind c
        if (far[b]) {
            out = b + 1 < (u32)NB ? far[b + 1] : absent_all;
            for (int e = 0; e < holders; ++e)
                if (lkey[e] > c && lgone[e] > out) out = lgone[e];
            for (int e = back; e < RANGE_LIST_CAP; ++e)
                if (lkey[e] > c && lgone[e] > out) out = lgone[e];
        }
        u64 d;
        if (out) {
            d = (u64)c + out;
        } else {
            u32 z = c;                                       // the candidate itself is in Z unless its successor is equal
            for (int e = 0; e < holders; ++e)
                if (lkey[e] <= c && lnext[e] > c && lkey[e] < z) z = lkey[e];
            d = (u64)(c - z);
        }
        if (d < bd || (d == bd && c < bk)) { bd = d; bk = c; }
    }
    wave_argmin(bd, bk);
    const int lane = tid & (WAVE - 1), wave = tid >> 6;
    u64* red = sm.red;
    if (lane == WAVE - 1) { red[wave] = bd; red[NW + wave] = bk; }
    __syncthreads();
    bd = red[0];
    bk = (u32)red[NW];
#pragma unroll
    for (int w = 1; w < NW; ++w) {
        const u64 od = red[w];
        const u32 ok = (u32)red[NW + w];
        if (od < bd || (od == bd && ok < bk)) { bd = od; bk = ok; }
    }
    best_d = bd;
    best_key = bk;
    return true;
}

template <int NT, int ITEMS, class CT>
struct RangeSearch {
    static constexpr bool PREDICTED = false;
    __device__ __forceinline__ static void run(const Smem& sm, const Rows& rw, const WinVal& wv, const InstInfo& ii, bool hot,
                                               const u32 (&lo)[ROWS_PER_THREAD<NT>], const u32 (&hi)[ROWS_PER_THREAD<NT>],
                                               Partial* __restrict__ out)
    {
        Partial r;
        r.wait = U64_MAX;
        r.brel = 0;
        if (wv.Elast >= wv.A) {
            bool done = false;
            if (hot && !(ii.range >> 31)) {                  // `gone` and `next` as positive 32-bit numbers
                u32 key;
                done = zl_range_bucket_search<NT, ITEMS, CT>(sm, rw, wv, ii.thr, lo, hi, r.wait, key);
                if (done) r.brel = r.wait == U64_MAX ? 0 : wv.A + key;
            }
            if (!done) { r.wait = U64_MAX; r.brel = DEFERRED_WINDOW; }
        }
        __syncthreads();                          // everyone is done with LDS before the next window
        if (threadIdx.x == 0) *out = r;
    }
};

// The fast range search over all windows; windows it cannot take are marked for
// zl_range_window_kernel.
template <int NT, int ITEMS, class CT>
__global__ __launch_bounds__(NT, 4) void zl_range_fast_kernel(
    const i64* __restrict__ ts, i64 B, int P, int R,
    const InstInfo* __restrict__ info, const CT* __restrict__ cross, int stride,
    const u32* __restrict__ winstart, const WinVal* __restrict__ winval, int max_win, u32 groups, u32 groups_inv,
    Partial* __restrict__ partial)
{
    using H = HotCfg<NT, ITEMS, false>;
    __shared__ __align__(16) unsigned char smem[H::BYTES];
    const Smem sm = carve_hot<NT, ITEMS>(smem);
    window_pairs<NT, ITEMS, CT, RangeSearch<NT, ITEMS, CT>>(sm, ts, nullptr, B, P, R, info, cross, stride, winstart,
                                                           winval, max_win, groups, groups_inv, partial);
}

// Instances of at most CAP_WIDE entries: one workgroup each.
template <int NT, int ITEMS>
__global__ __launch_bounds__(NT) void zl_range_instance_kernel(
    const i64* __restrict__ ts, int P, int R,
    i64* __restrict__ barrier, int* __restrict__ iters, i64* __restrict__ dmin,
    int* __restrict__ status)
{
    using C = WinCfg<NT, ITEMS>;
    __shared__ __align__(16) unsigned char smem[C::BYTES];
    const Smem sm = carve<NT, ITEMS>(smem);
    const int tid = threadIdx.x;
    const i64 b = blockIdx.x;
    const i64* __restrict__ inst = ts + b * (i64)P * R;
    i64 mn = INT64_MAX, mxf = INT64_MIN, mxl = INT64_MIN;
    for (int p = tid; p < P; p += NT) {
        const i64 f = inst[(size_t)p * R], l = inst[(size_t)p * R + R - 1];
        mn = f < mn ? f : mn;
        mxf = f > mxf ? f : mxf;
        mxl = l > mxl ? l : mxl;
    }
    i64 base, first_max, last_max;
    block_bounds<NT>(mn, mxf, mxl, (i64*)sm.red, base, first_max, last_max);
    const u64 range = (u64)last_max - (u64)base;
    const u64 thr = (u64)first_max - (u64)base;
    u32 flags = 0;
    u64 best_d = U64_MAX, best_rel = 0;
    int bad = 0;
    if (range >= 0xffffffffull) {
        flags |= EBSP_STATUS_UNSUPPORTED;
    } else {
        Rows rw;
        rw.inst = inst; rw.le = nullptr; rw.iv = nullptr; rw.P = P; rw.R = R; rw.base = (u64)base;
        rw.cr = nullptr; rw.narrow = false; rw.stride = 0; rw.k0 = rw.k1 = 0;
        zl_range_window<NT, ITEMS>(sm, rw, thr, 0ull, range, best_d, best_rel, bad);
    }
    if (__syncthreads_or(bad)) flags |= EBSP_STATUS_UNSORTED;
    if (best_d == U64_MAX) { best_d = 0; best_rel = 0; }
    const i64 bar = (i64)((u64)base + best_rel);
    if (tid == 0) {
        barrier[b] = bar;
        dmin[b] = (i64)best_d;
        if (status) status[b] = (int)flags;
    }
    for (int p = tid; p < P; p += NT)
        iters[b * (i64)P + p] = zl_iters(inst + (size_t)p * R, R, bar);
}

// The windows zl_range_fast_kernel marked: the sort-based search.  A fixed grid; every
// workgroup looks through its share of the window results for the marks and handles the
// marked windows one after the other.  Results go to `partial` (reduced by
// zl_finish_kernel like those of the summed-wait search).
template <int NT, int ITEMS>
__global__ __launch_bounds__(NT) void zl_range_window_kernel(
    const i64* __restrict__ ts, i64 B, int P, int R,
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
            const i64 b = pick / (u32)max_win;
            const InstInfo ii = info[b];
            const WinPos w = locate_window(b, (int)(pick % (u32)max_win), ii, ts, nullptr, nullptr, P, R, cross, narrow,
                                           stride, winstart, winval, max_win);
            Partial r;
            r.wait = U64_MAX;
            r.brel = 0;
            int bad = 0;
            bool fits = true;
            if (ii.range >= 0xffffffffull) fits = false;
            else if (w.valid) zl_range_window<NT, ITEMS>(sm, w.rw, ii.thr, w.A, w.Elast, r.wait, r.brel, bad);
            bad = __syncthreads_or(bad);
            if (threadIdx.x == 0) {
                partial[pick] = r;
                if (status && (bad || !fits))
                    atomicOr(status + b, (bad ? (int)EBSP_STATUS_UNSORTED : 0) | (fits ? 0 : (int)EBSP_STATUS_UNSUPPORTED));
            }
        }
    }
}

// zl_iters for the multi-window path: reduce the instance's window results
// (first minimum: smaller wait, then earlier barrier), then count iterations.
template <int NT>
__global__ __launch_bounds__(NT) void zl_finish_kernel(
    const i64* __restrict__ ts, const i64* __restrict__ le, const i64* __restrict__ iv, int P, int R,
    const InstInfo* __restrict__ info, const Partial* __restrict__ partial, int max_win,
    i64* __restrict__ barrier, int* __restrict__ iters, i64* __restrict__ wait)
{
    __shared__ u64 red[2 * (NT / WAVE)];
    constexpr int NW = NT / WAVE;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid >> 6;
    const u32 pblocks = (u32)(P + NT - 1) / NT;
    const i64 b = blockIdx.x / pblocks;
    const int pblk = (int)(blockIdx.x % pblocks);
    const InstInfo ii = info[b];
    u64 bw = U64_MAX, bb = U64_MAX;
    const Partial* pp = partial + b * (i64)max_win;
    for (int j = tid; j < (int)ii.nwin; j += NT) {
        const Partial r = pp[j];
        if (r.wait < bw || (r.wait == bw && r.brel < bb)) { bw = r.wait; bb = r.brel; }
    }
    wave_argmin(bw, bb);
    if (lane == WAVE - 1) { red[wave] = bw; red[NW + wave] = bb; }
    __syncthreads();
    bw = red[0]; bb = red[NW];
#pragma unroll
    for (int w = 1; w < NW; ++w) {
        const u64 ow = red[w], ob = red[NW + w];
        if (ow < bw || (ow == bw && ob < bb)) { bw = ow; bb = ob; }
    }
    if (bw == U64_MAX) bb = 0;
    const i64 bar = (i64)((u64)ii.base + bb);
    if (pblk == 0 && tid == 0) { barrier[b] = bar; wait[b] = (i64)bw; }
    const int p = pblk * NT + tid;
    if (p < P)
        iters[b * (i64)P + p] = zl_iters_of(ts ? ts + b * (i64)P * R : nullptr, le ? le + b * (i64)P : nullptr,
                                            iv ? iv + b * (i64)P : nullptr, p, R, bar);
}

// Plain streaming copy of n 16-byte words: the yardstick that HBM byte counters
// and achieved bandwidth of the other kernels are read against.
__global__ __launch_bounds__(256) void zl_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, i64 n)
{
    const i64 stride = (i64)gridDim.x * blockDim.x;
    for (i64 i = (i64)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// ---------------------------------------------------------------------------
// Host side.

thread_local char g_err[256] = "";

int fail(int code, const char* msg)
{
    snprintf(g_err, sizeof g_err, "%s", msg);
    return code;
}

enum KernelId { K_INSTANCE = 0, K_INSTANCE_GENERAL, K_BOUNDS, K_PARTITION, K_BINCOUNT, K_PLAN, K_WINDOW,
                K_WINDOW_GENERAL, K_FINISH, K_COPY, K_RANGE_INSTANCE, K_RANGE_WINDOW, K_PARTITION_PRED, K_RANGE_FAST, K_COUNT };
const char* const kKernelNames[K_COUNT] = {
    "zl_instance_kernel", "zl_instance_general_kernel", "zl_bounds_kernel", "zl_partition_kernel",
    "zl_bincount_kernel", "zl_plan_kernel", "zl_window_kernel", "zl_window_general_kernel",
    "zl_finish_kernel", "zl_copy_kernel", "zl_range_instance_kernel", "zl_range_window_kernel",
    "zl_partition_pred_kernel", "zl_range_fast_kernel"};

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Shape-dependent sizes of the multi-window path.
struct Tuning {          // 0: choose by shape
    int window_cap;
    int single_max;
    int window_fill;
};
Tuning g_tune = {0, 0, 0};

struct Plan {
    bool multi;
    int cap;           // records per window workgroup
    int fill;          // most entries of a window (unless a single fine bin holds more)
    int part_stored, part_pred;   // groups of rows whose column sums the partition kernels write (stored / predicted rows)
    int bins;          // fine bins per instance
    int stride;        // bins + 1 crossing indices per row
    int max_win;       // windows per instance <= max_win
    bool narrow;       // crossing indices fit 16 bits
    size_t off_info, off_seg, off_cross, off_part, off_below, off_winstart, off_winval, off_partial, off_rowpar, bytes;
};

// single_limit: the most entries one workgroup takes whole on the path the plan is for;
// list_room: windows leave a quarter or more of the workgroup's records free (the fast range search keeps its short list there)
bool make_plan(i64 B, int P, int R, Plan& pl, int single_limit = SINGLE_MAX, bool list_room = false)
{
    if (B < 0 || P < 1 || R < 1) return false;
    const i64 n = (i64)P * (i64)R;
    if (n >= (1ll << 31)) return false;
    memset(&pl, 0, sizeof pl);
    int single_max = g_tune.single_max > 0 ? g_tune.single_max : SINGLE_MAX;
    if (single_max > single_limit) single_max = single_limit;
    pl.multi = n > single_max;
    if (!pl.multi) return true;
    // the per-window cost has a term proportional to P: larger windows for more rows
    pl.cap = g_tune.window_cap > 0 ? g_tune.window_cap : (P >= 512 ? 8192 : 4096);
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
                 char* wsp, int* status, hipStream_t st)
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
    const i64 nrows = B * (i64)P;
    const i64 kblocks = (pl.stride + 255) / 256;
    const i64 widest = pl.part_stored > pl.part_pred ? pl.part_stored : pl.part_pred;
    if (kblocks * B > 0x7fffffffll || widest * B > 0x7fffffffll) return fail(EBSP_ERR_SHAPE, "batch too large for one call");
    LAUNCH(K_BOUNDS, (zl_bounds_kernel<256>), dim3((unsigned)B), dim3(256), ts, le, iv, P, R, pl.bins, info, segtab, rowpar, status);
    int part_rows;                                    // rows of partial column sums per instance (0: none, count from cross)
    if (pred) {
        part_rows = pl.part_pred;
        if (pl.narrow)
            LAUNCH(K_PARTITION_PRED, zl_partition_pred_kernel<unsigned short>, dim3((unsigned)(kblocks * B), (unsigned)part_rows),
                   dim3(256), le, iv, P, R, info, segtab, (unsigned short*)cross, pl.stride, part);
        else
            LAUNCH(K_PARTITION_PRED, zl_partition_pred_kernel<u32>, dim3((unsigned)(kblocks * B), (unsigned)part_rows),
                   dim3(256), le, iv, P, R, info, segtab, (u32*)cross, pl.stride, part);
    } else if (pl.part_stored > 0) {
        part_rows = pl.part_stored;
        if (pl.narrow)
            LAUNCH(K_PARTITION, zl_partition_sum_kernel<unsigned short>, dim3((unsigned)(B * part_rows)), dim3(PART_ROWS * WAVE),
                   ts, P, R, part_rows, info, segtab, (unsigned short*)cross, pl.stride, part, status);
        else
            LAUNCH(K_PARTITION, zl_partition_sum_kernel<u32>, dim3((unsigned)(B * part_rows)), dim3(PART_ROWS * WAVE),
                   ts, P, R, part_rows, info, segtab, (u32*)cross, pl.stride, part, status);
    } else {
        part_rows = 0;
        if (pl.narrow)
            LAUNCH(K_PARTITION, (zl_partition_kernel<256, unsigned short>), dim3((unsigned)((nrows + 3) / 4)), dim3(256),
                   ts, nrows, P, R, info, segtab, (unsigned short*)cross, pl.stride, status);
        else
            LAUNCH(K_PARTITION, (zl_partition_kernel<256, u32>), dim3((unsigned)((nrows + 3) / 4)), dim3(256),
                   ts, nrows, P, R, info, segtab, (u32*)cross, pl.stride, status);
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
        LAUNCH(K_PLAN, (zl_plan_kernel<256, 1024>), dim3((unsigned)B), dim3(256), info, segtab, below, pl.stride, winstart, winval,
               pl.max_win, (u32)pl.fill, (u32)(pl.cap / 8));
    else
        LAUNCH(K_PLAN, (zl_plan_kernel<1024, 4096>), dim3((unsigned)B), dim3(1024), info, segtab, below, pl.stride, winstart, winval,
               pl.max_win, (u32)pl.fill, (u32)(pl.cap / 8));
    return EBSP_OK;
}

// The rows are either stored (ts != nullptr) or predicted: t[p][i] = le[p] + (i + 1) * iv[p] (ts == nullptr).
int run_batch(const i64* ts, const i64* le, const i64* iv, i64 B, int P, int R,
              i64* barrier, int* iters, i64* wait, int* status,
              void* workspace, size_t workspace_bytes, hipStream_t st)
{
    Plan pl;
    if (!make_plan(B, P, R, pl)) return fail(EBSP_ERR_SHAPE, "invalid shape: need B >= 0, P >= 1, R >= 1, P*R < 2^31");
    if (B == 0) return EBSP_OK;
    const bool pred = ts == nullptr;
    if ((pred && (!le || !iv)) || !barrier || !iters || !wait)
        return fail(EBSP_ERR_NULL, "the input arrays, barrier, iters and wait must not be NULL");
    if (B > 0x7fffffffll) return fail(EBSP_ERR_SHAPE, "B must be below 2^31");
    const int n = P * R;

    if (!pl.multi) {
        const int rshift = (R & (R - 1)) == 0 ? __builtin_ctz((unsigned)R) : -1;
        const dim3 grid((unsigned)B);
#define LAUNCH_INSTANCE(NT_, ITEMS_)                                                                        \
    do {                                                                                                    \
        if (pred) LAUNCH(K_INSTANCE, (zl_instance_kernel<NT_, ITEMS_, true>), grid, dim3(NT_), ts, le, iv, P, R, rshift, \
                         barrier, iters, wait, status);                                                     \
        else LAUNCH(K_INSTANCE, (zl_instance_kernel<NT_, ITEMS_, false>), grid, dim3(NT_), ts, le, iv, P, R, rshift, \
                    barrier, iters, wait, status);                                                          \
    } while (0)
        if (n <= 256) LAUNCH_INSTANCE(128, 2);
        else if (n <= 1024) LAUNCH_INSTANCE(256, 4);
        else if (n <= 4096) LAUNCH_INSTANCE(512, 8);
        else LAUNCH_INSTANCE(1024, 16);
#undef LAUNCH_INSTANCE
        LAUNCH(K_INSTANCE_GENERAL, (zl_instance_general_kernel<LARGE_NT, LARGE_ITEMS>),
               dim3((unsigned)(B < GENERAL_GRID ? B : GENERAL_GRID)), dim3(LARGE_NT),
               ts, le, iv, B, P, R, barrier, iters, wait, status);
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

    if (int rc = plan_windows(pl, ts, le, iv, B, P, R, wsp, status, st)) return rc;
    const i64 pblocks = (P + 255) / 256;
    if (pblocks * B > 0x7fffffffll) return fail(EBSP_ERR_SHAPE, "batch too large for one call");
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
    LAUNCH(K_WINDOW_GENERAL, (zl_window_general_kernel<LARGE_NT, LARGE_ITEMS>),
           dim3((unsigned)(total_win < GENERAL_GRID ? total_win : GENERAL_GRID)), dim3(LARGE_NT),
           ts, le, iv, B, P, R, info, cross, pl.narrow, pl.stride, winstart, winval, pl.max_win, partial, status);
    LAUNCH(K_FINISH, (zl_finish_kernel<256>), dim3((unsigned)(pblocks * B)), dim3(256),
           ts, le, iv, P, R, info, partial, pl.max_win, barrier, iters, wait);
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

    if (int rc = plan_windows(pl, ts, nullptr, nullptr, B, P, R, wsp, status, st)) return rc;
    const i64 pblocks = (P + 255) / 256;
    if (pblocks * B > 0x7fffffffll) return fail(EBSP_ERR_SHAPE, "batch too large for one call");
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
           ts, nullptr, nullptr, P, R, info, partial, pl.max_win, barrier, iters, dmin);
    return EBSP_OK;
}

}  // namespace

extern "C" {

size_t ebsp_zipline_workspace_bytes(int64_t B, int32_t P, int32_t R)
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
    g_tune.window_cap = window_cap;
    g_tune.single_max = single_max;
    g_tune.window_fill = window_fill;
    return EBSP_OK;
}

int ebsp_zipline_copy_probe(const void* src, void* dst, size_t bytes, void* stream)
{
    if (!src || !dst) return fail(EBSP_ERR_NULL, "src and dst must not be NULL");
    if (bytes == 0 || bytes % 16 != 0 || (((uintptr_t)src | (uintptr_t)dst) & 15u))
        return fail(EBSP_ERR_SHAPE, "copy probe needs a positive multiple of 16 bytes and 16-byte aligned pointers");
    hipStream_t st = (hipStream_t)stream;
    const i64 n = (i64)(bytes / 16);
    i64 blocks = (n + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    LAUNCH(K_COPY, zl_copy_kernel, dim3((unsigned)blocks), dim3(256), (const uint4*)src, (uint4*)dst, n);
    if (g_prof.on && g_prof.calls < g_prof.max_calls) ++g_prof.calls;
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

// The search under the objective max(Z) - min(Z).
// Part of the ZipLine library (see zipline.hip); device code for gfx950.
#pragma once
#include "zl_window.h"

namespace {

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
// An interval is at most 2^32 - 2 wide (keys and the NEVER mark share 32 bits); a `next`
// beyond the interval is as good as NEVER inside it.  `gone` reaches back before the
// interval: it fits 32 bits when the instance's value spread does (below 2^32 - 1);
// otherwise (FAR) it is kept in 64 bits, its upper half in a third plane.
constexpr u32 NEVER = 0xffffffffu;
constexpr u64 RANGE_PIECE_MAX = 0xfffffffeull;          // widest interval searched in one go

template <bool FAR> struct Gone { using type = u32; static constexpr u32 never = NEVER; };
template <> struct Gone<true> { using type = u64; static constexpr u64 never = U64_MAX; };

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
template <int NT, bool FAR>
__device__ __forceinline__ int zl_range_gather(const Smem& sm, const Rows& rw, u64 a, u64 el, bool lx, bool rx,
                                               int cap, typename Gone<FAR>::type& absent, int& bad)
{
    using G = typename Gone<FAR>::type;
    const u64 width = el - a;
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
                const G gone = lo > 0 ? (G)(a - rw.rel(p, lo - 1)) : Gone<FAR>::never;
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
            u32 next = NEVER;
            G gone = 0;
            if (i + 1 < (u32)rw.R) {
                const i64 nxt = src[1];
                bad |= (nxt < cur);
                const u64 nrel = (u64)nxt - rw.base - a;
                next = FAR && nrel > width ? NEVER : (u32)nrel;
            }
            if (i == rowlo[l]) {                  // the row's first entry inside the interval
                gone = Gone<FAR>::never;
                if (i > 0) {
                    const i64 prv = src[-1];
                    bad |= (cur < prv);
                    gone = (G)(a - ((u64)prv - rw.base));
                }
            }
            const int slot = phys(total + e);
            sm.recs[slot] = (u64)(u32)(rel - a) | ((u64)next << 32);
            sm.dhi[slot] = (u32)gone;
            if (FAR) sm.ext[slot] = (u32)((u64)gone >> 32);
        }
        total += (int)chunk;
        __syncthreads();
    }
    return total;
}

// The search over the sorted entries [0, total); thread t owns positions
// [t*items, (t+1)*items).  Returns the first minimum (d, key); d == U64_MAX: none.
template <int NT, bool FAR>
__device__ __forceinline__ void zl_range_scan_argmin(const Smem& sm, int items, int total, u64 a, u64 thr,
                                                     typename Gone<FAR>::type absent_all, u64& best_d, u32& best_key)
{
    using GT = typename Gone<FAR>::type;
    u64* recs = sm.recs;
    auto gone = [&](int slot) -> GT { return FAR ? (GT)(((u64)sm.ext[slot] << 32) | sm.dhi[slot]) : (GT)sm.dhi[slot]; };
    GT* mirror = (GT*)sm.cnt;                    // NT of them (the counter plane holds 2*NT words at least)
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
    GT far = 0;
    for (int q = q0; q < qe; ++q) { const GT g = gone(phys(q)); far = g > far ? g : far; }
    mirror[NT - 1 - tid] = far;
    __syncthreads();
    const GT mv = mirror[tid];
    __syncthreads();
    const GT behind_m = block_excl_scan_op<GT, NT>(mv, (GT*)sm.red, OpMax());   // for thread NT-1-tid
    mirror[NT - 1 - tid] = behind_m;
    __syncthreads();                              // also: every M is in place
    GT G = mirror[tid];
    G = absent_all > G ? absent_all : G;

    u64 bd = U64_MAX;
    u32 bq = 0xffffffffu, bk = 0;
    for (int q = qe - 1; q >= q0; --q) {          // right to left: G covers the positions behind q
        const u32 key = (u32)recs[phys(q)];
        if (a + key >= thr && G != Gone<FAR>::never) {
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
        const GT g = gone(phys(q));
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

// One interval [A, Elast]: gather, sort, search.  An interval wider than RANGE_PIECE_MAX
// (FAR only) or with more than CAP_WIDE entries is walked in pieces that do fit, the latter
// cut by bisection on the value (every piece is searched on its own: what a piece needs from outside it
// are the neighbouring entries of its rows, which the gather reads); a single value
// that alone occurs more than CAP_WIDE times is one candidate and is evaluated
// directly from the rows.  (bd, bb) is updated with the first minimum found.
template <int NT, int ITEMS, bool FAR>
__device__ __forceinline__ void zl_range_window(const Smem& sm, const Rows& rw, u64 thr, u64 A, u64 Elast,
                                                u64& bd, u64& bb, int& bad)
{
    using C = WinCfg<NT, ITEMS>;
    using GT = typename Gone<FAR>::type;
    constexpr int CAPW = C::CAP_WIDE;
    u64 a = A;
    bool lx = true;
    for (;;) {
        u64 el = Elast;
        bool rx = true;
        if (FAR && el - a > RANGE_PIECE_MAX) { el = a + RANGE_PIECE_MAX; rx = false; }
        GT absent = 0;
        int total = zl_range_gather<NT, FAR>(sm, rw, a, el, lx, rx, CAPW, absent, bad);
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
                total = zl_range_gather<NT, FAR>(sm, rw, a, el, lx, false, CAPW, absent, bad);
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
            const GT absent_all = block_reduce<GT, NT>(absent, (GT*)sm.red, OpMax());   // also orders the record writes
            if (total > 0) {
                const int items = (total + NT - 1) / NT;
                fill_sentinels<NT>(sm.recs, total, items);
                __syncthreads();
                zl_sort<NT, ITEMS, true, FAR>(sm, items, bit_length(el - a));
                u64 d;
                u32 key;
                zl_range_scan_argmin<NT, FAR>(sm, items, total, a, thr, absent_all, d, key);
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
template <int NT> constexpr int RANGE_LIST_WORDS = 4 * 2 * NT;      // the short list: 2*NT entries of four words


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
    u32* reach = (u32*)(sm.red - H::NB);                    // NB words, later M
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
    const int total = zl_place_rows<NT, CT, false, true>(sm, rw, rw.base + a, H::CAP, lo, hi, unused, absent);
    best_d = U64_MAX;
    best_key = 0;
    if (total > H::CAP - 2 * RANGE_LIST_CAP) return false;
    if (total == 0) return true;
    const LinearMap bucket = linear_map((u32)(wv.Elast - a), NB, wv.scale ? wv.scale : 1u, wv.inv52);
    const u32* words = (const u32*)recs;                    // the source words
    auto read_entry = [&](u32 src, u32& key, u32& next, u32& gone) {     // an entry through its source word
        const u32 at = src & SRC_INDEX;
        const bool inner = (src & SRC_SEGMENT) && !(src & SRC_ROW);   // has a predecessor before the window
        const bool last = (src & SRC_LAST) != 0;
        const u32 cur = *(const u32*)(bytes + (at << 3));
        const u32 nxt = *(const u32*)(bytes + ((at + (last ? 0u : 1u)) << 3));
        const u32 prv = *(const u32*)(bytes + ((at - (inner ? 1u : 0u)) << 3));
        key = cur - start;
        next = last ? NEVER : nxt - start;
        gone = inner ? start - prv : 0u;
    };
    // sweep 2: reach, far and the entry count of every bucket; the keys stay in registers.  The three
    // words of every entry of a batch are asked for before any of them is used.
    u32 key[ITEMS];
    constexpr int RB = ITEMS;                               // (measured: all of a thread's entries at once, 2 % over batches of 8)
    static_assert(ITEMS % RB == 0, "batches must tile the items");
#pragma unroll
    for (int g = 0; g < ITEMS; g += RB) {
#pragma unroll
        for (int j = 0; j < RB; ++j) key[g + j] = 0;
        if (g * NT < total) {
            u32 src[RB];
            u32 cur[RB], nxt[RB], prv[RB];
#pragma unroll
            for (int j = 0; j < RB; ++j) {
                const int q = (g + j) * NT + tid;
                src[j] = q < total ? words[q] : (SRC_ROW | SRC_LAST);          // beyond the end: entry 0 alone, harmless
            }
#pragma unroll
            for (int j = 0; j < RB; ++j) {
                const u32 at = src[j] & SRC_INDEX;
                const u32 up = src[j] >> 29;                                   // the marks: row, segment, last
                const u32 inner = (up >> 1) & ~up & 1u;                       // has a predecessor before the window
                const u32 more = ~(up >> 2) & 1u;                              // not the row's last entry
                cur[j] = *(const u32*)(bytes + (at << 3));
                nxt[j] = *(const u32*)(bytes + ((at + more) << 3));
                prv[j] = *(const u32*)(bytes + ((at - inner) << 3));
            }
#pragma unroll
            for (int j = 0; j < RB; ++j) {
                const int q = (g + j) * NT + tid;
                const u32 up = src[j] >> 29;
                const bool inner = ((up >> 1) & ~up & 1u) != 0, last = ((up >> 2) & 1u) != 0;
                key[g + j] = cur[j] - start;
                if (q < total) {
                    const u32 b = bucket(key[g + j]);
                    atomicAdd(&flag[b], 1u);
                    atomicMax(&reach[b], last ? NEVER : nxt[j] - start);
                    if (inner && start != prv[j]) atomicMax(&far[b], start - prv[j]);
                }
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
    u32* mirror = (u32*)recs + ((total + 3) & ~3);          // NT words behind the source words
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
        read_entry(words[lslot[e] & 0xffffu], lkey[e], lnext[e], lgone[e]);
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
__global__ __launch_bounds__(NT, (NT > 512 ? 4 : 6)) void zl_range_fast_kernel(
    const i64* __restrict__ ts, i64 B, int P, int R,
    const InstInfo* __restrict__ info, const CT* __restrict__ cross, int stride,
    const u32* __restrict__ winstart, const WinVal* __restrict__ winval, int max_win, u32 groups, u32 groups_inv,
    Partial* __restrict__ partial)
{
    // the source words of at most CAP - 2 * (2*NT) entries, then the short list
    using L = WinHot<NT, ITEMS, false, RANGE_LIST_WORDS<NT> - 4 * NT>;
    __shared__ __align__(16) unsigned char smem[L::BYTES];
    const Smem sm = L::carve(smem);
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
    Rows rw;
    rw.inst = inst; rw.le = nullptr; rw.iv = nullptr; rw.P = P; rw.R = R; rw.base = (u64)base;
    rw.cr = nullptr; rw.narrow = false; rw.wide = false; rw.stride = 0; rw.k0 = rw.k1 = 0;
    if (range > RANGE_PIECE_MAX) zl_range_window<NT, ITEMS, true>(sm, rw, thr, 0ull, range, best_d, best_rel, bad);
    else zl_range_window<NT, ITEMS, false>(sm, rw, thr, 0ull, range, best_d, best_rel, bad);
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
            if (w.valid) {
                if (ii.range > RANGE_PIECE_MAX) zl_range_window<NT, ITEMS, true>(sm, w.rw, ii.thr, w.A, w.Elast, r.wait, r.brel, bad);
                else zl_range_window<NT, ITEMS, false>(sm, w.rw, ii.thr, w.A, w.Elast, r.wait, r.brel, bad);
            }
            bad = __syncthreads_or(bad);
            if (threadIdx.x == 0) {
                partial[pick] = r;
                if (status && bad) atomicOr(status + b, (int)EBSP_STATUS_UNSORTED);
            }
        }
    }
}

}  // namespace

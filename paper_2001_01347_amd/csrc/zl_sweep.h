// The frontier sweep: the summed-wait search of stored rows in one pass over the input.
// Part of the ZipLine library (see zipline.hip); device code for gfx950.
#pragma once
#include "zl_finish.h"

namespace {

// Algorithm 2 sweeps the merged, sorted timestamps once.  Here one workgroup sweeps a slice of
// an instance's value range, a window at a time, without any table that says where a window
// crosses the rows:
//   * every row keeps a cursor (the first entry the sweep has not passed).  A plan gives row p a
//     run of n_p consecutive record slots, n_p in proportion to the row's entries per unit of time
//     in what is left of the slice, so that all runs reach about equally far ahead;
//   * a step loads, for every row, the n_p entries from its cursor on (lanes that follow each
//     other read entries that follow each other).  The frontier F is the smallest last loaded
//     value over the rows that have more entries behind their run: every entry <= F of every row
//     is then in registers, so the window [A, F] is complete.  Its entries are consumed, exactly
//     as a window of the other kernels is searched: (key, delta) into value buckets (zl_delta and
//     the counting sort of zl_sort), bucket prefix sums (zl_scan), bounds that drop the buckets
//     which cannot hold the minimum, and the exact evaluation of what is left (zl_argmin).  The
//     cursors move past the consumed entries, W0 = P*A - S(A-) is carried to the next window
//     (no row is looked at again), and so is the best upper bound, which prunes later windows;
//   * a window never holds more than the workgroup's records, whatever the data: there is nothing
//     to defer.  Buckets are 2^sh wide (exact bounds by shifts).  Where a surviving bucket is too
//     deep to evaluate entry by entry (clustered or massively tied values), or holds a step of
//     2^31 or more, the step is taken again with a smaller F; at sh = 0 a bucket is one value and
//     is evaluated from its prefix sum alone.
// Slices of an instance are the fine bins of zl_bounds' map (about equal entry counts); a row's
// index range in a slice comes from a guided search for the slice's two ends, the same in the two
// workgroups that share an end, so the ranges tile the row.  Every loaded neighbour pair is
// compared as 64-bit values: a row that is not sorted raises EBSP_STATUS_UNSORTED.

constexpr u32 SWEEP_SPAN_MAX = 1u << 30;       // widest window of one step (keys and deltas stay below 2^31)
constexpr u32 KEY_NONE = 0xffffffffu;          // a record that is not part of the window
constexpr u32 KEY_STALE = 0xfffffffeu;         // an entry equal to an earlier frontier that was not loaded then: passed over, adds nothing
constexpr u32 SWEEP_DEEP = 64;                 // deepest bucket that is evaluated entry by entry
constexpr u32 SLOT_LAST = 1u << 15, SLOT_ROW = SLOT_LAST - 1;     // a slot's half word: its row, and whether it ends the row's run
constexpr u32 SLOT_GONE = 0x3ffffu;            // list-slot field of a bucket that was dropped

template <int NT, int ITEMS>
struct SweepCfg {
    static constexpr int NW = NT / WAVE;
    static constexpr int CAP = NT * ITEMS;       // record slots of a workgroup
    static constexpr int NB = CAP / 4;           // value buckets of a window (a power of two)
    static constexpr int BPT = NB / NT;          // buckets a thread scans
    static constexpr int LOG_NB = CAP == 16384 ? 12 : (CAP == 8192 ? 11 : (CAP == 4096 ? 10 : 9));
    static constexpr int LIST = NB / 2;          // entries of the surviving buckets
    static constexpr int RED_WORDS = 4 * NW + 8;
    static constexpr int MISC_WORDS = 16 + NW;
    static_assert((1 << LOG_NB) == NB && BPT * NT == NB && BPT % 2 == 0, "2048 to 16384 slots, an even number of buckets per thread");
    static_assert(CAP * 2 <= NB * 8, "the plan's slot markers lie over one set of bucket words");
    static_assert(ITEMS % 2 == 0, "two slots per register");
    __host__ __device__ static constexpr size_t bytes(int P)
    {
        return (size_t)(P + 2) * 16 + (size_t)NB * 8 * 2 + (size_t)LIST * 8 + (size_t)RED_WORDS * 8 + (size_t)CAP * 2 +
               (size_t)MISC_WORDS * 4;
    }
};

struct SweepSm {
    uint4* rowinfo;   // [P + 2]: x = offset (into the instance) of the row's first entry not consumed, y = first slot of its run,
                      //          z = offset behind its last entry of the slice, w = offset of its entry 0.  Entry P: {0, slots in use, 0, 0}
    u64* hist;        // [NB] per bucket: entries << 46 | sum of deltas; after the scan: first list slot << 46 | sum before the
                      // bucket.  Then [NB] more: all zero, except that they take the sums of the deltas of 2^31 or more when a
                      // step has such (after the scan: their sum before the bucket), and the plan's markers for a while.
    u64* recs;        // [LIST] (key, delta) of the surviving buckets' entries
    u32* slotmap;     // [CAP / 2] the row of every slot (and whether the slot ends its row's run), two slots per word; the words of
                      // a thread's items follow each other
    u64* red;         // [RED_WORDS]
    u32* misc;        // [MISC_WORDS]
};
enum { M_LIVE = 0, M_OFFEND = 1, M_FLAGS = 2, M_STALE = 3, M_CARRY = 16 };
constexpr u32 FLAG_NEG = 1, FLAG_GIANT = 2;

template <int NT, int ITEMS>
__device__ __forceinline__ SweepSm carve_sweep(unsigned char* smem, int P)
{
    using C = SweepCfg<NT, ITEMS>;
    SweepSm s;
    s.rowinfo = (uint4*)smem;
    s.hist = (u64*)(smem + (size_t)(P + 2) * 16);
    s.recs = s.hist + 2 * C::NB;
    s.red = s.recs + C::LIST;
    s.slotmap = (u32*)(s.red + C::RED_WORDS);
    s.misc = s.slotmap + C::CAP / 2;
    return s;
}

// First index of a sorted row whose value (relative to base) is >= v, R if none: a guess from the row's
// ends, a few doubling steps away from it, then bisection.  Every probe lies inside the row, and on any
// data the result x has row[x-1] < v <= row[x] (where those entries exist).
__device__ __forceinline__ u32 sweep_search(const i64* __restrict__ row, u32 R, u64 base, u64 v)
{
    const u64 f = (u64)row[0] - base, l = (u64)row[R - 1] - base;
    if (v <= f) return 0;
    if (v > l) return R;
    u32 lo = 0, hi = R - 1;                          // row[lo] < v <= row[hi] from here on
    if (hi - lo > 2) {
        const double frac = (double)(v - f) / (double)(l - f);
        u32 g = (u32)(frac * (double)(R - 1));
        g = g < 1 ? 1 : (g > R - 2 ? R - 2 : g);
        u32 step = 1;
        if ((u64)row[g] - base < v) {
            lo = g;
            while (hi - lo > step) {
                if ((u64)row[lo + step] - base < v) { lo += step; step *= 2; } else { hi = lo + step; break; }
            }
        } else {
            hi = g;
            while (hi - lo > step) {
                if ((u64)row[hi - step] - base >= v) { hi -= step; step *= 2; } else { lo = hi - step; break; }
            }
        }
    }
    while (hi - lo > 1) {
        const u32 m = lo + ((hi - lo) >> 1);
        if ((u64)row[m] - base < v) lo = m; else hi = m;
    }
    return hi;
}

// A thread's share (BPT consecutive words) of a set of bucket words back to zero.
template <int BPT>
__device__ __forceinline__ void zero_share(u64* words)
{
    uint4* z = (uint4*)(words + (size_t)threadIdx.x * BPT);
#pragma unroll
    for (int i = 0; i < BPT / 2; ++i) z[i] = make_uint4(0u, 0u, 0u, 0u);
}

// A value that is the same in every lane, moved to where such values live.
__device__ __forceinline__ u32 uniform(u32 x) { return (u32)__builtin_amdgcn_readfirstlane((int)x); }
__device__ __forceinline__ u64 uniform(u64 x) { return (u64)uniform((u32)x) | ((u64)uniform((u32)(x >> 32)) << 32); }

// The slot word of item j out of the four words that hold eight items.
__device__ __forceinline__ u32 slot_half(const uint4& w, int j)
{
    const u32 x = (j >> 1) == 0 ? w.x : ((j >> 1) == 1 ? w.y : ((j >> 1) == 2 ? w.z : w.w));
    return (x >> (16 * (j & 1))) & 0xffffu;
}

// Smallest shift that puts the values below x into NB buckets.
template <int LOG_NB>
__device__ __forceinline__ u32 shift_for(u64 x)
{
    const int bl = bit_length(x > 0 ? x - 1 : 0);
    return bl > LOG_NB ? (u32)(bl - LOG_NB) : 0u;
}

// A plan: slots for the rows that still have entries in the slice.  With `remaining` entries left in all
// rows together: every row gets them all if they fit; otherwise one slot each, and the other slots in
// proportion to rate_p = entries left / (last value of the row in the slice - A + 1).  Writes rowinfo[].y
// and the slot -> row map (slotmap), and returns how far ahead of A the runs are expected to reach (the same
// in every thread).  `scratch` is a set of bucket words that holds nothing; the other set is used too (and left
// at zero again).
template <int NT, int ITEMS, int RPT>     // RPT: the most rows a thread plans for
__device__ __forceinline__ u64 sweep_plan(const SweepSm& sm, u64* scratch, const i64* __restrict__ inst, int P, u64 a_abs, u32 remaining,
                                          u64 left)
{
    using C = SweepCfg<NT, ITEMS>;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid >> 6;
    const int chunk = (P + NT - 1) / NT;                      // consecutive rows per thread
    const int p0 = tid * chunk, p1 = p0 + chunk < P ? p0 + chunk : P;
    unsigned short* marker = (unsigned short*)scratch;        // CAP markers: row + 1 at the first slot of its run
    u64* rates = sm.hist;                                     // P <= NB words (zero again at the end)
    constexpr u64 RATE_MAX = 1ull << 50;                      // rates are 24.40 fixed point, capped
    const bool all_fit = remaining <= (u32)C::CAP;
    __syncthreads();                                          // (the bucket words have just been cleared by other threads)
    u64 rate_sum = 0;
    u32 active = 0;
    for (int p = p0; p < p1; ++p) {
        const uint4 ri = sm.rowinfo[p];
        const u32 rem = ri.z - ri.x;
        u64 rate = 0;
        if (rem && !all_fit) {
            const i64 span = (i64)((u64)inst[ri.z - 1] - a_abs) + 1;
            const double r = (double)rem * 1099511627776.0 / (double)(span > 0 ? span : 1);
            rate = r < (double)RATE_MAX ? (u64)r + 1 : RATE_MAX;
        }
        rates[p] = rate;
        rate_sum += rate;
        active += rem ? 1u : 0u;
    }
    rate_sum = uniform(block_reduce<u64, NT>(rate_sum, sm.red, OpAdd()));
    active = uniform(block_reduce<u32, NT>(active, (u32*)sm.red, OpAdd()));
    const u64 spare = (u64)C::CAP - active;                   // P <= CAP / 4, so this is most of the slots
    u32 mine = 0;
    u32 nrow[RPT];                                            // (chunk <= RPT)
#pragma unroll
    for (int c = 0; c < RPT; ++c) {
        const int p = p0 + c;
        u32 n = 0;
        if (p < p1) {
            const uint4 ri = sm.rowinfo[p];
            const u32 rem = ri.z - ri.x;
            n = rem;
            if (rem && !all_fit) {
                const u64 extra = rate_sum ? rates[p] * spare / rate_sum : 0;    // < 2^50 * 2^14: no overflow; the floors add up to <= spare
                n = 1u + (u32)extra;
                n = n < rem ? n : rem;
            }
        }
        nrow[c] = n;
        mine += n;
    }
    u32 total;
    u32 off = block_excl_scan<u32, NT>(mine, (u32*)sm.red, total);
    total = uniform(total);
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) marker[(wave * ITEMS + j) * WAVE + lane] = 0;
    __syncthreads();
#pragma unroll
    for (int c = 0; c < RPT; ++c) {
        const int p = p0 + c;
        if (p < p1) {
            sm.rowinfo[p].y = off;
            if (nrow[c]) marker[off] = (unsigned short)(p + 1);
            off += nrow[c];
        }
    }
    if (tid == 0) sm.rowinfo[P] = make_uint4(0u, total, 0u, 0u);
    __syncthreads();
    // the row of every slot: the latest marker at or before it.  Inside a wave's 64 * ITEMS slots by lane
    // moves; the marker that is open at the wave's first slot comes from the waves before it.
    u32 run = 0;
    u32 found[ITEMS];
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const u32 slot = (u32)(wave * ITEMS + j) * WAVE + lane;
        u32 v = wave_scan((u32)marker[slot], OpMax());
        v = v > run ? v : run;
        run = (u32)__shfl((int)v, WAVE - 1, WAVE);
        found[j] = v;                                         // the latest marker inside the wave's range
    }
    u32* wmax = (u32*)sm.red;
    if (lane == 0) wmax[wave] = run;
    __syncthreads();
    u32 before = 0;
    for (int w = 0; w < wave; ++w) { const u32 x = wmax[w]; before = x > before ? x : before; }
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const u32 slot = (u32)(wave * ITEMS + j) * WAVE + lane;
        const u32 m = found[j] > before ? found[j] : before;
        u32 r = (u32)P;                                       // slots beyond the plan: the entry that is never active
        if (slot < total && m) {
            r = m - 1u;
            const bool ends = slot + 1 == total || (slot + 1 < (u32)C::CAP && marker[slot + 1] != 0);
            if (ends) r |= SLOT_LAST;
        }
        found[j] = r;
    }
#pragma unroll
    for (int j = 0; j < ITEMS; j += 2) sm.slotmap[tid * (ITEMS / 2) + (j >> 1)] = found[j] | (found[j + 1] << 16);
    __syncthreads();                                          // done with the markers: the words go back to zero
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) marker[(wave * ITEMS + j) * WAVE + lane] = 0;
    for (int p = p0; p < p1; ++p) rates[p] = 0;
    // how far the runs reach: spare slots / sum of the rates (in 24.40 fixed point), or the rest of the slice
    u64 reach = left;
    if (!all_fit && rate_sum) {
        const u64 h = (spare << 40) / rate_sum;
        reach = h < left ? h : left;
    }
    __syncthreads();
    return reach;
}

// The cursors move behind the consumed entries (bit j of `cons`: the thread's item j): the lane that holds a
// row's last consumed entry writes the row's new cursor.  Whether the slot after a wave's last one is consumed
// is read from misc[M_CARRY + wave + 1], which the next wave wrote before the last barrier.
template <int NT, int ITEMS>
__device__ __forceinline__ void sweep_move_cursors(const SweepSm& sm, u32 cons, u32 slot0)
{
    constexpr int NW = NT / WAVE;
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x >> 6;
    const uint4* words = (const uint4*)(sm.slotmap + (size_t)threadIdx.x * (ITEMS / 2));
    u64 m = __ballot(cons & 1u);
#pragma unroll 1
    for (int g = 0; g < ITEMS; g += 8) {
        const uint4 w = words[g >> 3];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int j = g + i;
            u64 mn;
            if (j + 1 < ITEMS) mn = __ballot((cons >> (j + 1)) & 1u);
            else mn = wave + 1 < NW ? (u64)sm.misc[M_CARRY + wave + 1] : 0ull;
            const u64 next = (m >> 1) | (mn << 63);
            const u32 half = slot_half(w, i);
            const u64 lastm = __ballot((half & SLOT_LAST) != 0);
            const u64 E = m & (lastm | ~next);
            if ((E >> lane) & 1ull) {
                uint4* rp = sm.rowinfo + (half & SLOT_ROW);
                const uint2 r2 = *(const uint2*)rp;
                rp->x = (r2.x - r2.y + slot0) + ((u32)j * WAVE + 1u);
            }
            m = mn;
        }
    }
}

// What a pass over the runs finds besides the keys.
struct PassFlags {
    u32 big;      // nonzero: some step is 2^31 or more
    u32 neg;      // top bit set: some entry lies before its predecessor
    u32 stale;    // entries before A in the thread's wave (each lane holds the wave's count)
};

// zl_delta: one pass over the runs.  Every loaded entry becomes a key (its value - A) and a delta (its value -
// its predecessor's, base for a row's entry 0).  LIST false: the keys <= F go into the buckets (count and
// delta into `hist`, a delta of 2^31 or more into `big` instead); returns the thread's consumed items as a bit
// mask (keys <= F, and the entries before A: in sorted rows repeats of an earlier frontier, which are passed
// over).  LIST true: the items of `cons` whose bucket survived go into the list.  `take` false: no key is taken.
template <int NT, int ITEMS, bool LIST>
__device__ __forceinline__ u32 sweep_pass(const SweepSm& sm, const i64* __restrict__ inst, u64 base, u64 a_abs, u32 F, u32 sh,
                                          bool take, u32 slot0, u32 cons, PassFlags& fl)
{
    using C = SweepCfg<NT, ITEMS>;
    static_assert(ITEMS % 8 == 0, "eight items a batch");
    u64* hist = sm.hist;
    u64* big = sm.hist + C::NB;
    u32 out = 0;
    constexpr int BATCH = 8;
    const uint4* words = (const uint4*)(sm.slotmap + (size_t)threadIdx.x * (ITEMS / 2));
#pragma unroll 1
    for (int g = 0; g < ITEMS; g += BATCH) {
        i64 cv[BATCH], pv[BATCH];
        bool act[BATCH], head[BATCH];
        const uint4 w = words[g >> 3];
        const u32 sg = slot0 + (u32)g * WAVE;
#pragma unroll
        for (int j = 0; j < BATCH; ++j) {
            const uint4 ri = sm.rowinfo[slot_half(w, j) & SLOT_ROW];
            const u32 e = (ri.x - ri.y + sg) + (u32)j * WAVE;
            act[j] = e < ri.z && (!LIST || ((cons >> (g + j)) & 1u));
            head[j] = e <= ri.w;                                          // the row's entry 0: its predecessor is base
            const u32 ce = act[j] ? e : 0u;
            const u32 pe = act[j] && !head[j] ? e - 1u : ce;
            cv[j] = inst[ce];
            pv[j] = inst[pe];
        }
#pragma unroll
        for (int j = 0; j < BATCH; ++j) {
            const u64 c = (u64)cv[j];
            const u64 pr = act[j] && head[j] ? base : (u64)pv[j];
            const u64 rel = c - a_abs, d = c - pr;
            const bool okc = act[j] && take && (rel >> 32) == 0 && (u32)rel <= F;
            const u32 k = (u32)rel;
            if (!LIST) {
                const bool old = act[j] && (i64)rel < 0;
                const u32 an = (u32)(d >> 32) | ((u32)d >> 31);           // a step of 2^31 or more, or backwards
                fl.big |= an;
                fl.neg |= (u32)(d >> 32) | (old && d != 0 ? 0x80000000u : 0u);
                fl.stale += (u32)__popcll(__ballot(old));
                out |= (okc || old) ? 1u << (g + j) : 0u;
                if (okc) {
                    atomicAdd(&hist[k >> sh], (1ull << 46) | (an ? 0ull : (u64)(u32)d));
                    if (an) atomicAdd(&big[k >> sh], d);
                }
            } else if (okc) {
                const u32 bq = k >> sh;
                if ((u32)(hist[bq] >> 46) < SLOT_GONE) {
                    const u32 slot = (u32)(atomicAdd(&hist[bq], 1ull << 46) >> 46);
                    if (slot < (u32)C::LIST) sm.recs[slot] = (u64)k | (d << 32);
                }
            }
        }
    }
    return out;
}

// One workgroup per slice of an instance; the slice's best candidate goes to partial[b * nslices + s].
template <int NT, int ITEMS, int PMAX>       // PMAX: the most rows the workgroup's LDS is laid out for
__global__ __launch_bounds__(NT, NT == 256 ? 2 : 4) void zl_sweep_kernel(
    const i64* __restrict__ ts, i64 B, int P, int R, int nslices,
    const InstInfo* __restrict__ info, const SegEntry* __restrict__ segtab,
    Partial* __restrict__ partial, int* __restrict__ status)
{
    using C = SweepCfg<NT, ITEMS>;
    constexpr int NW = C::NW;
    static_assert(PMAX <= C::NB && PMAX < (int)SLOT_ROW && 4 * PMAX <= C::CAP, "rate words, row field, a slot for every row");
    static_assert(ITEMS <= 32, "one bit per item");
    __shared__ __align__(16) unsigned char sweep_smem[C::bytes(PMAX)];
    const SweepSm sm = carve_sweep<NT, ITEMS>(sweep_smem, P);
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid >> 6;
    const i64 b = blockIdx.x / (u32)nslices;
    const u32 s = blockIdx.x % (u32)nslices;
    if (b >= B) return;
    const InstInfo ii = info[b];
    Partial res;
    res.wait = U64_MAX;
    res.brel = 0;
    Partial* out = partial + b * (i64)nslices + s;
    if (s >= ii.nb || (ii.flags & EBSP_STATUS_UNSORTED)) {
        if (tid == 0) *out = res;
        return;
    }
    const i64* __restrict__ inst = ts + b * (i64)P * R;
    const u64 base = (u64)ii.base;
    u64* hist = sm.hist;                       // the bucket words
    u64* big = sm.hist + C::NB;                // all zero except while a step has deltas of 2^31 or more (and inside the plan)
    // the slice: values (relative to base) in [vs, ve)
    if (tid < 2) {
        const u32 k = s + (u32)tid;
        sm.red[tid] = k < ii.nb ? fine_bin_start(k, ii, segtab + b * (i64)SEGS) : ii.range + 1;
    }
    zero_share<C::BPT>(hist);
    zero_share<C::BPT>(big);
    __syncthreads();
    const bool first_slice = s == 0, last_slice = s + 1 == ii.nb;
    const u64 vs = first_slice ? 0ull : uniform(sm.red[0]), ve = last_slice ? ii.range + 1 : uniform(sm.red[1]);
    __syncthreads();

    // the rows' index ranges in the slice; W0 = sum_p (vs - last value of row p before the slice), a row that has
    // not begun standing at base
    u64 W0;
    u32 remaining;
    int bad;
    {
        u64 w0 = 0;
        u32 rem = 0;
        int wrong = 0;
        for (int p = tid; p < P; p += NT) {
            const i64* __restrict__ row = inst + (size_t)p * R;
            const u32 lo = first_slice ? 0u : sweep_search(row, (u32)R, base, vs);
            u32 hi = last_slice ? (u32)R : sweep_search(row, (u32)R, base, ve);
            if (hi < lo) { wrong = 1; hi = lo; }
            const u64 before = lo > 0 ? (u64)row[lo - 1] - base : 0ull;
            w0 += vs - before;
            const u32 r0 = (u32)p * (u32)R;
            sm.rowinfo[p] = make_uint4(r0 + lo, 0u, r0 + hi, r0);
            rem += hi - lo;
        }
        W0 = uniform(block_reduce<u64, NT>(w0, sm.red, OpAdd()));
        remaining = uniform(block_reduce<u32, NT>(rem, (u32*)sm.red, OpAdd()));
        bad = __syncthreads_or(wrong);
    }
    if (tid == 0) { sm.misc[M_LIVE] = 0; sm.misc[M_OFFEND] = 0xffffffffu; sm.misc[M_FLAGS] = 0; sm.misc[M_STALE] = 0; }

    u64 A = vs;                                   // first value of the window to come (relative to base)
    const u64 thr = ii.thr;
    const u64 PP = (u64)(u32)P;
    i64 UB = INT64_MAX;                           // best upper bound of the minimum so far
    u64 best_w = U64_MAX, best_c = U64_MAX;       // this thread's best candidate: wait, barrier relative to base
    bool replan = true;
    const u32 slot0 = (u32)(wave * ITEMS) * WAVE + lane;
    const u64 step_cap = 2ull * remaining + 64;   // sorted rows never come near it
    constexpr int RPT = (PMAX + NT - 1) / NT;     // rows whose frontier a thread looks up
    const int chunk = (P + NT - 1) / NT;
    const int rp0 = tid * chunk;
    constexpr u64 SMASK = (1ull << 46) - 1;       // low field of a bucket word

    for (u64 step = 0; remaining > 0 && !bad; ++step) {
        if (step > step_cap) { bad = 1; break; }
        if (replan) {
            sweep_plan<NT, ITEMS, RPT>(sm, big, inst, P, base + A, remaining, ve - A);
            replan = false;
        }
        const u64 a_abs = base + A;
        // ---- the frontier: the smallest last value of a run that entries follow (as F + 1; 0 says that such a run
        // ends before A, with entries equal to an earlier frontier that were not loaded when it passed: then nothing
        // but such entries can be passed over in this step); and the smallest value that is left at all
        u32 F1;
        u64 first_rel;
        {
            u32 fmin = SWEEP_SPAN_MAX + 1u;
            u64 cmin = U64_MAX;
#pragma unroll
            for (int c = 0; c < RPT; ++c) {
                const int p = rp0 + c;
                if (c < chunk && p < P) {
                    const uint4 ri = sm.rowinfo[p];
                    const u32 n = sm.rowinfo[p + 1].y - ri.y;
                    if (n && ri.x + n < ri.z) {
                        const u64 rel = (u64)inst[ri.x + n - 1] - a_abs;
                        const u32 f = (i64)rel < 0 ? 0u : ((rel >> 32) == 0 && (u32)rel < SWEEP_SPAN_MAX ? (u32)rel + 1u : SWEEP_SPAN_MAX + 1u);
                        fmin = f < fmin ? f : fmin;
                    }
                    if (ri.x < ri.z) {
                        const u64 rel = (u64)inst[ri.x] - base;
                        cmin = rel < cmin ? rel : cmin;
                    }
                }
            }
            fmin = wave_scan(fmin, OpMin());
            cmin = wave_scan(cmin, OpMin());
            if (lane == WAVE - 1) { ((u32*)sm.red)[wave] = fmin; sm.red[NW + wave] = cmin; }
            __syncthreads();                                              // B1 (also: the bucket words are zero, the plan is there)
            F1 = ((u32*)sm.red)[0];
            first_rel = sm.red[NW];
#pragma unroll
            for (int w = 1; w < NW; ++w) {
                const u32 x = ((u32*)sm.red)[w];
                const u64 y = sm.red[NW + w];
                F1 = x < F1 ? x : F1;
                first_rel = y < first_rel ? y : first_rel;
            }
            F1 = uniform(F1);
            first_rel = uniform(first_rel);
            if (ve - A < (u64)F1) F1 = (u32)(ve - A);                     // the slice ends there: no entry of it lies beyond
        }
        const u64 need64 = thr > A ? thr - A : 0ull;
        const u32 need = need64 > 0xffffffffull ? 0xffffffffu : (u32)need64;      // keys >= need are admissible

        // ---- the window [A, A + F]: its entries into the buckets, the buckets scanned and bounded.  Once more with a
        // smaller F where a surviving bucket cannot be evaluated entry by entry: up to before it, or (if it is the
        // first) that bucket alone, cut finer.
        u32 F = F1 ? F1 - 1u : 0u;
        u32 sh = 0, cons = 0, consumed = 0, stale = 0, live = 0;
        u64 dsum = 0;
        bool anyg = false;
        for (;;) {
            sh = shift_for<C::LOG_NB>((u64)F + 1);
            PassFlags pf;
            pf.big = pf.neg = pf.stale = 0;
            cons = sweep_pass<NT, ITEMS, false>(sm, inst, base, a_abs, F, sh, F1 != 0, slot0, 0u, pf);
            if (lane == 0) {
                sm.misc[M_CARRY + wave] = cons & 1u;                      // is the wave's first slot consumed
                if (pf.stale) atomicAdd(&sm.misc[M_STALE], pf.stale);
            }
            {
                u32 fl = (pf.neg >> 31) ? FLAG_NEG : 0u;
                fl |= pf.big ? FLAG_GIANT : 0u;
                if (fl) atomicOr(&sm.misc[M_FLAGS], fl);
            }
            __syncthreads();                                              // B2: the bucket words are complete
            const u32 flags = uniform(sm.misc[M_FLAGS]);
            stale = uniform(sm.misc[M_STALE]);
            if (flags & FLAG_NEG) { bad = 1; break; }
            anyg = (flags & FLAG_GIANT) != 0;
            if (F1 == 0) break;                                           // nothing but repeats of an earlier frontier
            // ---- zl_scan over the buckets, BPT per thread; bounds; which buckets survive
            u64 h[C::BPT], gg[C::BPT];
            {
                const uint4* h4 = (const uint4*)(hist + (size_t)tid * C::BPT);
#pragma unroll
                for (int i = 0; i < C::BPT / 2; ++i) {
                    const uint4 a = h4[i];
                    h[2 * i] = (u64)a.x | ((u64)a.y << 32);
                    h[2 * i + 1] = (u64)a.z | ((u64)a.w << 32);
                }
            }
            u64 tot = 0, gtot = 0;
#pragma unroll
            for (int i = 0; i < C::BPT; ++i) {
                gg[i] = anyg ? big[tid * C::BPT + i] : 0ull;
                tot += h[i];
                gtot += gg[i];
            }
            const u64 inc = wave_scan(tot, OpAdd());
            const u64 ginc = anyg ? wave_scan(gtot, OpAdd()) : 0ull;
            // smallest P*hi - E over the admissible buckets, E counted from the wave's first bucket
            i64 u = INT64_MAX;
            {
                u64 e = (inc - tot) & SMASK, ge = ginc - gtot;
#pragma unroll
                for (int i = 0; i < C::BPT; ++i) {
                    const u32 lo = (u32)(tid * C::BPT + i) << sh;
                    const u32 top = lo + ((1u << sh) - 1u);
                    const u32 hi = top < F ? top : F;
                    e += h[i] & SMASK;
                    ge += gg[i];
                    if ((h[i] >> 46) && lo >= need) {
                        const i64 x = (i64)(PP * hi - e - ge);
                        u = x < u ? x : u;
                    }
                }
            }
            u = wave_scan(u, OpMin());
            if (lane == WAVE - 1) { sm.red[wave] = inc; sm.red[NW + wave] = (u64)u; sm.red[2 * NW + wave] = ginc; }
            __syncthreads();                                              // Bs
            u64 hbase = 0, total = 0, gbase = 0, gsum = 0;
            i64 um = INT64_MAX;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const u64 xh = sm.red[w], xg = sm.red[2 * NW + w];
                const i64 uw = (i64)sm.red[NW + w];
                const i64 cand = uw == INT64_MAX ? uw : uw - (i64)(total & SMASK) - (i64)gsum;
                um = cand < um ? cand : um;
                if (w < wave) { hbase += xh; gbase += xg; }
                total += xh;
                gsum += xg;
            }
            hbase += inc - tot;
            gbase += ginc - gtot;
            total = uniform(total);
            gsum = uniform(gsum);
            um = (i64)uniform((u64)um);
            consumed = (u32)(total >> 46);
            dsum = (total & SMASK) + gsum;
            i64 ubn = UB;
            if (um != INT64_MAX) { const i64 x = um + (i64)W0; ubn = x < ubn ? x : ubn; }
            const i64 ubrel = ubn == INT64_MAX ? ubn : ubn - (i64)W0;
            {
                u64 e = hbase & SMASK, ge = gbase;
#pragma unroll
                for (int i = 0; i < C::BPT; ++i) {
                    const u32 lo = (u32)(tid * C::BPT + i) << sh;
                    const u32 top = lo + ((1u << sh) - 1u);
                    const u32 hi = top < F ? top : F;
                    const u32 c = (u32)(h[i] >> 46);
                    const u64 eb = e, gb = ge;
                    e += h[i] & SMASK;
                    ge += gg[i];
                    u32 at = SLOT_GONE;
                    if (sh == 0) {
                        // a bucket is one value: its prefix sum is the candidate's
                        if (c && lo >= need) {
                            const u64 w = PP * lo + W0 - e - ge;
                            const u64 cabs = A + lo;
                            if (w < best_w || (w == best_w && cabs < best_c)) { best_w = w; best_c = cabs; }
                        }
                    } else {
                        if (c && hi >= need && (i64)(PP * lo - e - ge) <= ubrel) {
                            if (c > SWEEP_DEEP || gg[i]) atomicMin(&sm.misc[M_OFFEND], (u32)(tid * C::BPT + i));
                            const u32 got = atomicAdd(&sm.misc[M_LIVE], c);
                            at = got < SLOT_GONE ? got : SLOT_GONE - 1u;
                        }
                        hist[tid * C::BPT + i] = eb | ((u64)at << 46);
                        if (anyg) big[tid * C::BPT + i] = gb;
                    }
                }
            }
            __syncthreads();                                              // B3
            if (sh == 0) { UB = ubn; break; }
            live = uniform(sm.misc[M_LIVE]);
            const u32 off = uniform(sm.misc[M_OFFEND]);
            if (off == 0xffffffffu && live <= (u32)C::LIST) { UB = ubn; break; }
            u32 fnew = off == 0xffffffffu ? F >> 1 : (off > 0 ? (off << sh) - 1u : (1u << sh) - 1u);
            if (fnew >= F) fnew = F >> 1;
            F = fnew;
            // everything of this pass is dropped (once everyone has read what it left)
            __syncthreads();
            if (tid == 0) { sm.misc[M_LIVE] = 0; sm.misc[M_OFFEND] = 0xffffffffu; sm.misc[M_FLAGS] = 0; sm.misc[M_STALE] = 0; }
            zero_share<C::BPT>(hist);
            if (anyg) zero_share<C::BPT>(big);
            live = 0;
            __syncthreads();
        }
        if (bad) break;

        if (F1 == 0) {
            // only repeats of an earlier frontier are passed over: the cursors move, A and W0 stay
            consumed = 0;
            if (stale == 0) { bad = 1; break; }                          // (sorted rows always have such entries here)
            sweep_move_cursors<NT, ITEMS>(sm, cons, slot0);
        } else if (consumed + stale == 0) {
            // nothing at or below F (a gap wider than a window): go on at the smallest value that is left
            if (first_rel == U64_MAX || first_rel <= A + F) { bad = 1; break; }   // only rows that are not sorted get here
            W0 += PP * (first_rel - A);
            A = first_rel;
        } else {
            // ---- zl_argmin: the entries of the surviving buckets are listed (their deltas formed again) and evaluated
            const bool listing = sh != 0 && live > 0;
            if (listing) {
                PassFlags unused;
                unused.big = unused.neg = unused.stale = 0;
                sweep_pass<NT, ITEMS, true>(sm, inst, base, a_abs, F, sh, true, slot0, cons, unused);
                __syncthreads();                                          // B4: the list is complete, the old cursors have been used
            }
            sweep_move_cursors<NT, ITEMS>(sm, cons, slot0);
            if (listing) {
                for (u32 q = tid; q < live; q += NT) {
                    const u32 k = (u32)sm.recs[q];
                    const u32 bq = k >> sh;
                    const u64 hb = hist[bq];
                    u64 S = hb & SMASK;
                    if (anyg) S += big[bq];
                    for (u32 x = (u32)(hb >> 46); x-- > 0;) {             // the bucket's entries end at its slot field
                        const u64 r = sm.recs[x];
                        if (((u32)r >> sh) != bq) break;
                        S += ((u32)r <= k) ? r >> 32 : 0ull;
                    }
                    if (k >= need) {
                        const u64 w = PP * k + W0 - S;
                        const u64 cabs = A + k;
                        if (w < best_w || (w == best_w && cabs < best_c)) { best_w = w; best_c = cabs; }
                    }
                }
            }
            W0 += PP * ((u64)F + 1) - dsum;
            A += (u64)F + 1;
        }
        remaining -= consumed + stale < remaining ? consumed + stale : remaining;
        // a new plan where the runs have grown uneven (rows ending, speeds changing), and for the last entries
        if (remaining > 0 && (2 * (consumed + stale) < (u32)C::CAP)) replan = true;
        __syncthreads();                                                  // end of the step: cursors written, list and words read
        if (tid == 0) { sm.misc[M_LIVE] = 0; sm.misc[M_OFFEND] = 0xffffffffu; sm.misc[M_FLAGS] = 0; sm.misc[M_STALE] = 0; }
        zero_share<C::BPT>(hist);
        if (anyg) zero_share<C::BPT>(big);
    }

    bad = __syncthreads_or(bad);
    if (bad) {
        if (tid == 0) {
            if (status) atomicOr(status + b, (int)EBSP_STATUS_UNSORTED);
            *out = res;
        }
        return;
    }
    // first minimum over the workgroup
    wave_argmin(best_w, best_c);
    if (lane == WAVE - 1) { sm.red[wave] = best_w; sm.red[NW + wave] = best_c; }
    __syncthreads();
    if (tid == 0) {
        u64 bw = sm.red[0], bc = sm.red[NW];
        for (int w = 1; w < NW; ++w) {
            const u64 ow = sm.red[w], oc = sm.red[NW + w];
            if (ow < bw || (ow == bw && oc < bc)) { bw = ow; bc = oc; }
        }
        res.wait = bw;
        res.brel = bw == U64_MAX ? 0 : bc;
        *out = res;
    }
}

// The slices' candidates -> barrier and wait of the instance (first minimum), then zl_iters: per row the
// number of entries <= barrier by bisection.
template <int NT>
__global__ __launch_bounds__(NT) void zl_sweep_finish_kernel(
    const i64* __restrict__ ts, int P, int R, int nslices, const InstInfo* __restrict__ info,
    const Partial* __restrict__ partial, i64* __restrict__ barrier, int* __restrict__ iters, i64* __restrict__ wait)
{
    const u32 pblocks = (u32)(P + NT - 1) / NT;
    const i64 b = blockIdx.x / pblocks;
    const int p = (int)(blockIdx.x % pblocks) * NT + (int)threadIdx.x;
    const InstInfo ii = info[b];
    const Partial* pp = partial + b * (i64)nslices;
    u64 bw = U64_MAX, bb = 0;
    const u32 n = ii.nb < (u32)nslices ? ii.nb : (u32)nslices;
    for (u32 j = 0; j < n; ++j) {                 // few slices: every thread looks through them
        const Partial r = pp[j];
        if (r.wait < bw || (r.wait == bw && r.wait != U64_MAX && r.brel < bb)) { bw = r.wait; bb = r.brel; }
    }
    const i64 bar = (i64)((u64)ii.base + bb);
    if (blockIdx.x % pblocks == 0 && threadIdx.x == 0) { barrier[b] = bar; wait[b] = (i64)bw; }
    if (p < P) iters[b * (i64)P + p] = zl_iters(ts + (b * (i64)P + p) * (i64)R, R, bar);
}

}  // namespace

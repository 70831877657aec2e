// The frontier sweep: the summed-wait search of stored rows in one pass over the input.
// Part of the ZipLine library (see zipline.hip); device code for gfx950.
#pragma once
#include "zl_finish.h"

namespace {

// Algorithm 2 sweeps the merged, sorted timestamps once.  Here one workgroup sweeps a slice of
// an instance's value range, a window at a time, without any table that says where a window
// crosses the rows, and every cache line of the input is asked for as a whole:
//   * every row keeps a cursor (the first entry the sweep has not passed).  A plan gives row p a
//     run of n_p lines (16 entries, 128 bytes, aligned in memory) from the line of its cursor on,
//     n_p chosen from the row's entries per unit of time in what is left of the slice, so that all
//     runs reach about equally far ahead of the cursors;
//   * the frontier F is the smallest last value of a run over the rows that have more entries
//     behind their run (one probe per row): every entry <= F of every row lies in a run, so the
//     window [A, F] is complete.  A step streams the runs once, sixteen lanes a line: an entry's
//     predecessor is the lane before it, its key (value - A) and delta go into value buckets
//     (zl_delta and the counting sort of zl_sort) and are not kept.  Then bucket prefix sums
//     (zl_scan), bounds that drop the buckets which cannot hold the minimum, and - only where
//     buckets survive - a second stream over the runs that lists their entries for the exact
//     evaluation (zl_argmin).  The cursors move past the consumed entries, W0 = P*A - S(A-) is
//     carried to the next window (no row is looked at again), and so is the best upper bound,
//     which prunes later windows (the slices of an instance share theirs through a word in memory);
//   * a window never holds more than the plan's lines, whatever the data: there is nothing to
//     defer.  Buckets are 2^sh wide (exact bounds by shifts).  Where a surviving bucket is too
//     deep to evaluate entry by entry (clustered or massively tied values), or the window holds a
//     step of 2^31 or more, the window is taken again with a smaller F; a window of one value
//     (F = 0) needs no buckets at all: its entries are counted and their deltas summed in 64 bits.
// Slices of an instance are the fine bins of zl_bounds' map (about equal entry counts); a row's
// index range in a slice comes from a guided search for the slice's two ends, the same in the two
// workgroups that share an end, so the ranges tile the row.  Every loaded neighbour pair is
// compared as 64-bit values: a row that is not sorted raises EBSP_STATUS_UNSORTED.

constexpr u32 SWEEP_SPAN_MAX = 1u << 30;       // widest window of one step (keys and deltas stay below 2^31)
constexpr u32 SWEEP_DEEP = 64;                 // deepest bucket that is evaluated entry by entry
constexpr u32 SLOT_GONE = 0x3ffffu;            // list-slot field of a bucket that was dropped
constexpr int LINE = 16;                       // entries of a line
constexpr int SWEEP_BATCH = 8;                 // lines a lane group has in flight

constexpr int log2_of(int x) { return x <= 1 ? 0 : 1 + log2_of(x / 2); }

template <int NT, int CAPL_, int NB_, int LIST_>
struct SweepCfg {
    static constexpr int NW = NT / WAVE;
    static constexpr int CAPL = CAPL_;           // lines of a plan
    static constexpr int CAP = CAPL * LINE;      // entries of a window at most (below 2^18: the count field of a bucket word)
    static constexpr int NB = NB_;               // value buckets of a window (a power of two)
    static constexpr int BPT = NB / NT;          // buckets a thread scans
    static constexpr int LOG_NB = log2_of(NB);
    static constexpr int LIST = LIST_;           // entries of the surviving buckets
    static constexpr int RED_WORDS = 4 * NW + 8;
    static constexpr int MISC_WORDS = 16;
    static_assert((1 << LOG_NB) == NB && BPT * NT == NB && BPT % 2 == 0, "a power of two, an even number of buckets per thread");
    static_assert(CAP < (1 << 18) && LIST < (int)SLOT_GONE, "18-bit count and slot fields");
    static_assert(CAPL % (4 * NW * SWEEP_BATCH) == 0, "whole rounds of the workgroup");
    __host__ __device__ static constexpr size_t bytes(int P)
    {
        return (size_t)(P + 2) * 16 + (size_t)((P + 3) / 4 * 4) * 4 + (size_t)NB * 8 + (size_t)LIST * 8 + (size_t)RED_WORDS * 8 +
               (size_t)CAPL * 2 + (size_t)MISC_WORDS * 4;
    }
};

struct SweepSm {
    uint4* rowinfo;   // [P + 2]: x = offset (into the instance) of the row's first entry not consumed, y = first line of its run,
                      //          z = offset behind its last entry of the slice, w = offset of the first entry of the line x lies
                      //          in (it may lie before the row, even before the instance).  Entry P: {0, lines in use, 0, 0}
    u32* curnew;      // [P] offset behind the row's last entry consumed in this step (0: none)
    u64* hist;        // [NB] per bucket: entries << 46 | sum of deltas; after the scan: first list slot << 46 | sum before the
                      // bucket.  Between steps all zero; the plan keeps the rows' rates there for a while.
    u64* recs;        // [LIST] (key, delta) of the surviving buckets' entries
    u64* red;         // [RED_WORDS]
    unsigned short* linemap;   // [CAPL] the row of every line of the plan
    u32* misc;        // [MISC_WORDS]
};
enum { M_LIVE = 0, M_OFFEND = 1, M_FLAGS = 2, M_STALE = 3, M_GIANT = 4 };
constexpr u32 FLAG_NEG = 1, FLAG_GIANT = 2;

template <class C>
__device__ __forceinline__ SweepSm carve_sweep(unsigned char* smem, int P)
{
    SweepSm s;
    s.rowinfo = (uint4*)smem;
    s.curnew = (u32*)(smem + (size_t)(P + 2) * 16);
    s.hist = (u64*)(s.curnew + (P + 3) / 4 * 4);
    s.recs = s.hist + C::NB;
    s.red = s.recs + C::LIST;
    s.linemap = (unsigned short*)(s.red + C::RED_WORDS);
    s.misc = (u32*)(s.linemap + C::CAPL);
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

// Smallest shift that puts the values below x into NB buckets.
template <int LOG_NB>
__device__ __forceinline__ u32 shift_for(u64 x)
{
    const int bl = bit_length(x > 0 ? x - 1 : 0);
    return bl > LOG_NB ? (u32)(bl - LOG_NB) : 0u;
}

// A plan: lines for the rows that still have entries in the slice.  Row p's run starts with the line of its
// cursor (o_p entries of that line lie before the cursor).  If every row's remaining entries fit, each row gets
// them all; otherwise the K = 16 * (lines - rows with entries) - sum of o_p entries that are free to give are
// shared in proportion to rate_p = entries left / (last value of the row in the slice - A + 1): row p gets
// floor((o_p + share_p) / 16) + 1 lines, which add up to no more than the plan has.  Writes rowinfo[].y,
// rowinfo[].w and the line -> row map.  `mis`: entries between the 128-byte boundary at or before the
// instance's first entry and that entry.
template <int NT, class C, int RPT>       // RPT: the most rows a thread plans for
__device__ __forceinline__ void sweep_plan(const SweepSm& sm, const i64* __restrict__ inst, int P, u32 lines, u32 mis, u64 a_abs)
{
    const int tid = threadIdx.x;
    const int chunk = (P + NT - 1) / NT;                      // consecutive rows per thread
    const int p0 = tid * chunk, p1 = p0 + chunk < P ? p0 + chunk : P;
    u64* rates = sm.hist;                                     // P <= NB words (zero again at the end)
    constexpr u64 RATE_MAX = 1ull << 46;                      // rates are 24.40 fixed point, capped
    __syncthreads();                                          // (the bucket words have just been cleared by other threads)
    u64 rate_sum = 0;
    u64 counts = 0;                                           // rows with entries | sum of o_p << 12 | lines for everything << 28
    for (int p = p0; p < p1; ++p) {
        const uint4 ri = sm.rowinfo[p];
        const u32 rem = ri.z - ri.x;
        u64 rate = 0;
        if (rem) {
            const u32 o = (ri.x + mis) & (LINE - 1);
            const i64 span = (i64)((u64)inst[ri.z - 1] - a_abs) + 1;
            const double r = (double)rem * 1099511627776.0 / (double)(span > 0 ? span : 1);
            rate = r < (double)RATE_MAX ? (u64)r + 1 : RATE_MAX;
            counts += 1ull | ((u64)o << 12) | ((u64)((o + rem + LINE - 1) / LINE) << 28);
        }
        rates[p] = rate;
        rate_sum += rate;
    }
    rate_sum = uniform(block_reduce<u64, NT>(rate_sum, sm.red, OpAdd()));
    counts = uniform(block_reduce<u64, NT>(counts, sm.red, OpAdd()));
    const u32 active = (u32)counts & 0xfffu, osum = (u32)(counts >> 12) & 0xffffu;
    const bool all_fit = (counts >> 28) <= (u64)lines;
    const u64 K = (u64)LINE * (lines - active) - osum;                        // P <= lines / 2, so this is positive
    u32 mine = 0;
    u32 nrow[RPT];                                            // (chunk <= RPT)
#pragma unroll
    for (int c = 0; c < RPT; ++c) {
        const int p = p0 + c;
        u32 n = 0;
        if (p < p1) {
            const uint4 ri = sm.rowinfo[p];
            const u32 rem = ri.z - ri.x;
            if (rem) {
                const u32 o = (ri.x + mis) & (LINE - 1);
                n = (o + rem + LINE - 1) / LINE;
                if (!all_fit) {
                    const u64 share = rate_sum ? rates[p] * K / rate_sum : 0;     // < 2^46 * 2^17: no overflow
                    const u64 m = (o + share) / LINE + 1;
                    n = m < n ? (u32)m : n;
                }
            }
        }
        nrow[c] = n;
        mine += n;
    }
    u32 total;
    u32 off = block_excl_scan<u32, NT>(mine, (u32*)sm.red, total);
    total = uniform(total);
#pragma unroll
    for (int c = 0; c < RPT; ++c) {
        const int p = p0 + c;
        if (p < p1) {
            uint4* rp = sm.rowinfo + p;
            const u32 cur = rp->x;
            rp->y = off;
            rp->w = cur - ((cur + mis) & (LINE - 1));
            for (u32 k = 0; k < nrow[c]; ++k) sm.linemap[off + k] = (unsigned short)p;
            off += nrow[c];
        }
    }
    if (tid == 0) sm.rowinfo[P] = make_uint4(0u, total, 0u, 0u);
    // the lines behind the plan's last one, up to a whole round of the workgroup, belong to "row P", which has no entries
    {
        constexpr u32 ROUND = 4u * (u32)(NT / WAVE) * (u32)SWEEP_BATCH;
        const u32 padded = (total + ROUND - 1) / ROUND * ROUND;
        for (u32 l = total + (u32)tid; l < padded; l += NT) sm.linemap[l] = (unsigned short)P;
    }
    for (int p = p0; p < p1; ++p) rates[p] = 0;
    __syncthreads();
}

// What a stream over the runs finds besides the keys.
struct PassOut {
    u32 giant;    // PASS_HIST: nonzero: some entry of the window lies 2^31 or more after its predecessor
    u32 neg;      // top bit set: some entry lies before its predecessor
    u32 stale;    // entries of the runs that lie before A although no window took them (each lane holds the wave's count)
    u32 count;    // PASS_ONE: the thread's entries of the window
    u64 dsum;     // PASS_ONE: the sum of their deltas
};
enum { PASS_HIST = 0, PASS_LIST = 1, PASS_ONE = 2, PASS_GIANT = 3 };

// zl_delta: one stream over the runs of a plan of T lines, sixteen lanes a line.  Every loaded entry becomes a key
// (its value - A) and a delta (its value - its predecessor's, base for a row's entry 0): the predecessor is the
// lane before, or (a line's first entry) loaded by itself.  Entries before the row's cursor are only predecessors.
// PASS_HIST: the keys <= F go into the buckets (count and delta; a delta of 2^31 or more raises po.giant and the window
// has to be taken again: PASS_GIANT then finds the smallest key with such a delta, into misc[M_GIANT]); the entries
// of the window and those before A ("stale": in sorted rows repeats of an earlier
// frontier that lay behind their run then) are consumed: curnew[] takes the offset behind each row's last one.
// PASS_LIST: the keys <= F whose bucket survived go into the list.  PASS_ONE (F = 0): the entries of the window are
// counted and their deltas summed; consumed as in PASS_HIST.  `take` false: no key is taken (stale entries only).
template <int NT, class C, int MODE>
__device__ __forceinline__ void sweep_pass(const SweepSm& sm, const i64* __restrict__ inst, int R, u64 base, u64 a_abs, u32 F, u32 sh,
                                           bool take, u32 T, PassOut& po)
{
    constexpr int NW = C::NW;
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x >> 6;
    const u32 sub = (u32)lane & (LINE - 1), grp = (u32)lane >> 4;
    u64* hist = sm.hist;
#pragma unroll 1
    for (u32 q0 = 0; 4u * q0 < T; q0 += (u32)(NW * SWEEP_BATCH)) {
        i64 cv[SWEEP_BATCH], pv[SWEEP_BATCH];
        int ent[SWEEP_BATCH];           // the entry's offset, -1: none
        u32 rowf[SWEEP_BATCH];          // its row | before the cursor << 16 | the row's entry 0 << 17
#pragma unroll
        for (int j = 0; j < SWEEP_BATCH; ++j) {
            const u32 l = 4u * (q0 + (u32)(j * NW + wave)) + grp;          // (behind the plan's lines: row P, no entries)
            const u32 row = (u32)sm.linemap[l];
            const uint4 ri = sm.rowinfo[row];
            const int e = (int)ri.w + (int)((l - ri.y) * LINE + sub);
            const int rs = (int)(row * (u32)R);
            const bool ok = e >= rs && (u32)e < ri.z;
            ent[j] = ok ? e : -1;
            rowf[j] = row | ((u32)e < ri.x ? 1u << 16 : 0u) | (e == rs ? 1u << 17 : 0u);
            cv[j] = inst[ok ? e : 0];
            pv[j] = 0;
            if (ok && sub == 0 && e > rs) pv[j] = inst[e - 1];
        }
#pragma unroll
        for (int j = 0; j < SWEEP_BATCH; ++j) {
            const bool ok = ent[j] >= 0;
            const bool pre = (rowf[j] >> 16) & 1u, head = (rowf[j] >> 17) & 1u;
            const u64 c = (u64)cv[j];
            u64 pr = dpp_take<DPP_ROW_SHR1, 0xf>((u64)0, c);
            pr = sub == 0 ? (u64)pv[j] : pr;
            pr = head ? base : pr;
            const u64 rel = c - a_abs, d = c - pr;
            const bool old = ok && !pre && (i64)rel < 0;
            const bool in = ok && !pre && take && (rel >> 32) == 0 && (u32)rel <= F;
            const u32 k = (u32)rel;
            if (MODE == PASS_LIST) {
                if (in) {
                    const u32 bq = k >> sh;
                    if ((u32)(hist[bq] >> 46) < SLOT_GONE) {
                        const u32 slot = (u32)(atomicAdd(&hist[bq], 1ull << 46) >> 46);
                        if (slot < (u32)C::LIST) sm.recs[slot] = (u64)k | (d << 32);
                    }
                }
            } else if (MODE == PASS_GIANT) {
                if (in && (d >> 31) != 0) atomicMin(&sm.misc[M_GIANT], k);
            } else {
                po.neg |= (ok ? (u32)(d >> 32) : 0u) | (old && d != 0 ? 0x80000000u : 0u);
                po.stale += (u32)__popcll(__ballot(old));
                if (MODE == PASS_ONE) {
                    po.count += in ? 1u : 0u;
                    po.dsum += in ? d : 0ull;
                } else {
                    po.giant |= in ? (u32)(d >> 31) : 0u;                  // (a delta of 2^31 or more spoils its bucket: the window is taken again)
                    if (in) atomicAdd(&hist[k >> sh], (1ull << 46) | (u64)((u32)d & 0x7fffffffu));
                }
                const bool cons = in || old;
                const u64 m = __ballot(cons);
                if (cons && (sub == LINE - 1 || !((m >> (lane + 1)) & 1ull))) atomicMax(&sm.curnew[rowf[j] & 0xffffu], (u32)ent[j] + 1u);
            }
        }
    }
}

// One workgroup per slice of an instance; the slice's best candidate goes to partial[b * nslices + s].
// `lines`: lines of a plan, 2 * P <= lines <= CAPL.
template <int NT, int CAPL, int NBK, int LISTN, int PMAX>       // PMAX: the most rows the workgroup's LDS is laid out for
__global__ __launch_bounds__(NT, NT == 256 ? 2 : 4) void zl_sweep_kernel(
    const i64* __restrict__ ts, i64 B, int P, int R, int nslices, int lines,
    const InstInfo* __restrict__ info, const SegEntry* __restrict__ segtab, i64* __restrict__ best,
    Partial* __restrict__ partial, int* __restrict__ status)
{
    using C = SweepCfg<NT, CAPL, NBK, LISTN>;
    constexpr int NW = C::NW;
    static_assert(PMAX <= C::NB && PMAX < 0xffff && 2 * PMAX <= CAPL, "rate words, row field, lines for every row");
    __shared__ __align__(16) unsigned char sweep_smem[C::bytes(PMAX)];
    const SweepSm sm = carve_sweep<C>(sweep_smem, P);
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
    const u32 mis = (u32)(((uintptr_t)inst >> 3) & (LINE - 1));
    const u64 base = (u64)ii.base;
    u64* hist = sm.hist;                       // the bucket words
    // the slice: values (relative to base) in [vs, ve)
    if (tid < 2) {
        const u32 k = s + (u32)tid;
        sm.red[tid] = k < ii.nb ? fine_bin_start(k, ii, segtab + b * (i64)SEGS) : ii.range + 1;
    }
    zero_share<C::BPT>(hist);
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
            sm.rowinfo[p] = make_uint4(r0 + lo, 0u, r0 + hi, 0u);
            sm.curnew[p] = 0;
            rem += hi - lo;
        }
        W0 = uniform(block_reduce<u64, NT>(w0, sm.red, OpAdd()));
        remaining = uniform(block_reduce<u32, NT>(rem, (u32*)sm.red, OpAdd()));
        bad = __syncthreads_or(wrong);
    }
    if (tid == 0) { sm.misc[M_LIVE] = 0; sm.misc[M_OFFEND] = 0xffffffffu; sm.misc[M_FLAGS] = 0; sm.misc[M_STALE] = 0; sm.misc[M_GIANT] = 0xffffffffu; }

    u64 A = vs;                                   // first value of the window to come (relative to base)
    const u64 thr = ii.thr;
    const u64 PP = (u64)(u32)P;
    i64 UB = INT64_MAX;                           // best upper bound of the minimum so far
    u64 best_w = U64_MAX, best_c = U64_MAX;       // this thread's best candidate: wait, barrier relative to base
    const u64 step_cap = 2ull * remaining + 64;   // sorted rows never come near it
    constexpr int RPT = (PMAX + NT - 1) / NT;     // rows a thread plans for and whose frontier it looks up
    const int chunk = (P + NT - 1) / NT;
    const int rp0 = tid * chunk;
    constexpr u64 SMASK = (1ull << 46) - 1;       // low field of a bucket word

    for (u64 step = 0; remaining > 0 && !bad; ++step) {
        if (step > step_cap) { bad = 1; break; }
        const u64 a_abs = base + A;
        sweep_plan<NT, C, RPT>(sm, inst, P, (u32)lines, mis, a_abs);
        const u32 T = uniform(sm.rowinfo[P].y);
        // ---- the frontier: the smallest last value of a run that entries follow (as F + 1; 0 says that such a run
        // ends before A, with entries equal to an earlier frontier that lay behind their run when it passed: then
        // nothing but such entries can be passed over in this step); and the smallest value that is left at all
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
                    const u32 runend = ri.w + n * LINE;
                    if (n && (int)runend < (int)ri.z) {
                        const u64 rel = (u64)inst[runend - 1] - a_abs;
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
            // what the other slices of the instance have found bounds the minimum as well (any admissible candidate's wait does)
            if (tid == 0) sm.red[2 * NW] = (u64)__atomic_load_n(best + b, __ATOMIC_RELAXED);
            __syncthreads();                                              // B1
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
            const i64 shared = (i64)uniform(sm.red[2 * NW]);
            UB = shared < UB ? shared : UB;
            if (ve - A < (u64)F1) F1 = (u32)(ve - A);                     // the slice ends there: no entry of it lies beyond
        }
        const u64 need64 = thr > A ? thr - A : 0ull;
        const u32 need = need64 > 0xffffffffull ? 0xffffffffu : (u32)need64;      // keys >= need are admissible

        // ---- the window [A, A + F]: its entries into the buckets, the buckets scanned and bounded.  Once more with a
        // smaller F where a surviving bucket cannot be evaluated entry by entry (up to before it, or, if it is the
        // first, that bucket alone, cut finer) or where the window holds a step of 2^31 or more (up to before it).
        u32 F = F1 ? F1 - 1u : 0u;
        u32 sh = 0, consumed = 0, stale = 0, live = 0;
        u64 dsum = 0;
        const i64 ub_before = UB;
        for (;;) {
            sh = shift_for<C::LOG_NB>((u64)F + 1);
            PassOut po;
            po.giant = po.neg = po.stale = po.count = 0;
            po.dsum = 0;
            const bool one = F == 0 && F1 != 0;
            if (one) sweep_pass<NT, C, PASS_ONE>(sm, inst, R, base, a_abs, F, sh, true, T, po);
            else sweep_pass<NT, C, PASS_HIST>(sm, inst, R, base, a_abs, F, sh, F1 != 0, T, po);
            if (lane == 0 && po.stale) atomicAdd(&sm.misc[M_STALE], po.stale);
            if ((po.neg >> 31) || po.giant) atomicOr(&sm.misc[M_FLAGS], ((po.neg >> 31) ? FLAG_NEG : 0u) | (po.giant ? FLAG_GIANT : 0u));
            __syncthreads();                                              // B2: the bucket words are complete
            const u32 flags = uniform(sm.misc[M_FLAGS]);
            stale = uniform(sm.misc[M_STALE]);
            if (flags & FLAG_NEG) { bad = 1; break; }
            if (F1 == 0) break;                                           // nothing but repeats of an earlier frontier
            if (one) {
                // one value: all its entries at once
                consumed = uniform(block_reduce<u32, NT>(po.count, (u32*)sm.red, OpAdd()));
                dsum = uniform(block_reduce<u64, NT>(po.dsum, sm.red, OpAdd()));
                if (consumed && need == 0 && tid == 0) {
                    const u64 w = W0 - dsum;
                    if (w < best_w || (w == best_w && A < best_c)) { best_w = w; best_c = A; }
                }
                if (consumed && need == 0) { const i64 x = (i64)(W0 - dsum); UB = x < UB ? x : UB; }
                break;
            }
            if (flags & FLAG_GIANT) {
                // a step of 2^31 or more inside the window: up to before the first such, or that value alone
                PassOut unused;
                unused.giant = unused.neg = unused.stale = unused.count = 0;
                unused.dsum = 0;
                sweep_pass<NT, C, PASS_GIANT>(sm, inst, R, base, a_abs, F, sh, true, T, unused);
                __syncthreads();
                const u32 giant = uniform(sm.misc[M_GIANT]);
                F = giant != 0xffffffffu && giant ? giant - 1u : 0u;
                __syncthreads();
                if (tid == 0) { sm.misc[M_STALE] = 0; sm.misc[M_GIANT] = 0xffffffffu; sm.misc[M_FLAGS] = 0; }
                zero_share<C::BPT>(hist);
                for (int p = tid; p < P; p += NT) sm.curnew[p] = 0;
                __syncthreads();
                continue;
            }
            // ---- zl_scan over the buckets, BPT per thread; bounds; which buckets survive
            u64 h[C::BPT];
            {
                const uint4* h4 = (const uint4*)(hist + (size_t)tid * C::BPT);
#pragma unroll
                for (int i = 0; i < C::BPT / 2; ++i) {
                    const uint4 a = h4[i];
                    h[2 * i] = (u64)a.x | ((u64)a.y << 32);
                    h[2 * i + 1] = (u64)a.z | ((u64)a.w << 32);
                }
            }
            u64 tot = 0;
#pragma unroll
            for (int i = 0; i < C::BPT; ++i) tot += h[i];
            const u64 inc = wave_scan(tot, OpAdd());
            // smallest P*hi - E over the admissible buckets, E counted from the wave's first bucket
            i64 u = INT64_MAX;
            {
                u64 e = (inc - tot) & SMASK;
#pragma unroll
                for (int i = 0; i < C::BPT; ++i) {
                    const u32 lo = (u32)(tid * C::BPT + i) << sh;
                    const u32 top = lo + ((1u << sh) - 1u);
                    const u32 hi = top < F ? top : F;
                    e += h[i] & SMASK;
                    if ((h[i] >> 46) && lo >= need) {
                        const i64 x = (i64)(PP * hi - e);
                        u = x < u ? x : u;
                    }
                }
            }
            u = wave_scan(u, OpMin());
            if (lane == WAVE - 1) { sm.red[wave] = inc; sm.red[NW + wave] = (u64)u; }
            __syncthreads();                                              // Bs
            u64 hbase = 0, total = 0;
            i64 um = INT64_MAX;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const u64 xh = sm.red[w];
                const i64 uw = (i64)sm.red[NW + w];
                const i64 cand = uw == INT64_MAX ? uw : uw - (i64)(total & SMASK);
                um = cand < um ? cand : um;
                if (w < wave) hbase += xh;
                total += xh;
            }
            hbase += inc - tot;
            total = uniform(total);
            um = (i64)uniform((u64)um);
            consumed = (u32)(total >> 46);
            dsum = total & SMASK;
            i64 ubn = UB;
            if (um != INT64_MAX) { const i64 x = um + (i64)W0; ubn = x < ubn ? x : ubn; }
            const i64 ubrel = ubn == INT64_MAX ? ubn : ubn - (i64)W0;
            {
                u64 e = hbase & SMASK;
#pragma unroll
                for (int i = 0; i < C::BPT; ++i) {
                    const u32 lo = (u32)(tid * C::BPT + i) << sh;
                    const u32 top = lo + ((1u << sh) - 1u);
                    const u32 hi = top < F ? top : F;
                    const u32 c = (u32)(h[i] >> 46);
                    const u64 eb = e;
                    e += h[i] & SMASK;
                    u32 at = SLOT_GONE;
                    if (sh == 0) {
                        // a bucket is one value: its prefix sum is the candidate's
                        if (c && lo >= need) {
                            const u64 w = PP * lo + W0 - e;
                            const u64 cabs = A + lo;
                            if (w < best_w || (w == best_w && cabs < best_c)) { best_w = w; best_c = cabs; }
                        }
                    } else {
                        if (c && hi >= need && (i64)(PP * lo - e) <= ubrel) {
                            if (c > SWEEP_DEEP) atomicMin(&sm.misc[M_OFFEND], (u32)(tid * C::BPT + i));
                            const u32 got = atomicAdd(&sm.misc[M_LIVE], c);
                            at = got < SLOT_GONE ? got : SLOT_GONE - 1u;
                        }
                        hist[tid * C::BPT + i] = eb | ((u64)at << 46);
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
            if (tid == 0) { sm.misc[M_LIVE] = 0; sm.misc[M_OFFEND] = 0xffffffffu; sm.misc[M_STALE] = 0; }
            zero_share<C::BPT>(hist);
            for (int p = tid; p < P; p += NT) sm.curnew[p] = 0;
            live = 0;
            __syncthreads();
        }
        if (bad) break;

        if (F1 == 0) {
            // only repeats of an earlier frontier are passed over: the cursors move, A and W0 stay
            consumed = 0;
            if (stale == 0) { bad = 1; break; }                          // (sorted rows always have such entries here)
        } else if (consumed + stale == 0) {
            // nothing at or below F (a gap wider than a window): go on at the smallest value that is left
            if (first_rel == U64_MAX || first_rel <= A + F) { bad = 1; break; }   // only rows that are not sorted get here
            W0 += PP * (first_rel - A);
            A = first_rel;
        } else {
            // ---- zl_argmin: the entries of the surviving buckets are listed (their deltas formed again) and evaluated
            if (sh != 0 && live > 0) {
                PassOut unused;
                unused.giant = unused.neg = unused.stale = unused.count = 0;
                unused.dsum = 0;
                sweep_pass<NT, C, PASS_LIST>(sm, inst, R, base, a_abs, F, sh, true, T, unused);
                __syncthreads();                                          // B4: the list is complete
                for (u32 q = tid; q < live; q += NT) {
                    const u32 k = (u32)sm.recs[q];
                    const u32 bq = k >> sh;
                    const u64 hb = hist[bq];
                    u64 S = hb & SMASK;
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
        if (tid == 0 && UB < ub_before) atomicMin(best + b, UB);
        // the cursors move behind the consumed entries
        for (int p = tid; p < P; p += NT) {
            const u32 cn = sm.curnew[p];
            if (cn) {
                if (cn > sm.rowinfo[p].x) sm.rowinfo[p].x = cn;
                sm.curnew[p] = 0;
            }
        }
        __syncthreads();                                                  // end of the step: list and words read
        if (tid == 0) { sm.misc[M_LIVE] = 0; sm.misc[M_OFFEND] = 0xffffffffu; sm.misc[M_FLAGS] = 0; sm.misc[M_STALE] = 0; sm.misc[M_GIANT] = 0xffffffffu; }
        zero_share<C::BPT>(hist);
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

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
constexpr u32 KEY_STALE = 0xfffffffeu;         // an entry equal to the last frontier that was not loaded then: passed over, adds nothing
constexpr u32 SWEEP_DROPPED = 0x80000000u;
constexpr u32 SWEEP_DEEP = 64;                 // deepest bucket that is evaluated entry by entry
constexpr u32 SLOT_FIRST = 1u << 30, SLOT_LAST = 1u << 31, SLOT_ROW = SLOT_FIRST - 1;

template <int NT, int ITEMS>
struct SweepCfg {
    static constexpr int NW = NT / WAVE;
    static constexpr int CAP = NT * ITEMS;       // record slots of a workgroup
    static constexpr int BPT = 4;                // buckets a thread scans
    static constexpr int NB = NT * BPT;          // value buckets of a window (a power of two)
    static constexpr int LOG_NB = NT == 1024 ? 12 : (NT == 512 ? 11 : 10);
    static constexpr int LIST = NB;              // entries of the surviving buckets
    static constexpr int RED_WORDS = 4 * NW + 8;
    static constexpr int MISC_WORDS = 16 + NW;
    static_assert((1 << LOG_NB) == NB, "NT is 256, 512 or 1024");
    static_assert(CAP * 2 <= NB * 8, "the plan's slot markers lie over the bucket words");
    __host__ __device__ static constexpr size_t bytes(int P)
    {
        return (size_t)(P + 2) * 16 + (size_t)NB * 8 * 2 + (size_t)LIST * 8 + (size_t)RED_WORDS * 8 + (size_t)NB * 4 +
               (size_t)MISC_WORDS * 4;
    }
};

struct SweepSm {
    uint4* rowinfo;   // [P + 2]: x = offset (into the instance) of the row's first entry not consumed, y = first slot of its run,
                      //          z = offset behind its last entry of the slice, w = offset of its entry 0.  Entry P: {0, slots in use, 0, 0}
    u64* hist;        // [NB] per bucket: entries << 46 | sum of deltas; after the scan: first list slot << 46 | sum before the bucket
    u64* hist2;       // [NB] per bucket: sum of the deltas of 2^31 or more; after the scan: their sum before the bucket
    u64* recs;        // [LIST] (key, delta) of the surviving buckets' entries
    u64* red;         // [RED_WORDS]
    u32* cnt;         // [NB] list slot of a surviving bucket's next entry, or SWEEP_DROPPED
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
    s.hist2 = s.hist + C::NB;
    s.recs = s.hist2 + C::NB;
    s.red = s.recs + C::LIST;
    s.cnt = (u32*)(s.red + C::RED_WORDS);
    s.misc = s.cnt + C::NB;
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

// A plan: slots for the rows that still have entries in the slice.  With `remaining` entries left in all
// rows together: every row gets them all if they fit; otherwise one slot each, and the other slots in
// proportion to rate_p = entries left / (last value of the row in the slice - A + 1).  Writes rowinfo[].y
// and the slot -> row map (slotrow), returns the number of slots in use (the same in every thread).
template <int NT, int ITEMS>
__device__ __forceinline__ u32 sweep_plan(const SweepSm& sm, const i64* __restrict__ inst, int P, u64 a_abs, u32 remaining,
                                          u32 (&slotrow)[ITEMS])
{
    using C = SweepCfg<NT, ITEMS>;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid >> 6;
    const int chunk = (P + NT - 1) / NT;                      // consecutive rows per thread
    const int p0 = tid * chunk, p1 = p0 + chunk < P ? p0 + chunk : P;
    u32* rown = sm.cnt;                                       // P <= NB words: the rows' slot counts
    unsigned short* marker = (unsigned short*)sm.hist;        // CAP markers: row + 1 at the first slot of its run
    constexpr u64 RATE_MAX = 1ull << 50;                      // rates are 24.40 fixed point, capped
    const bool all_fit = remaining <= (u32)C::CAP;
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
        sm.hist2[p] = rate;                                   // (free between steps; P <= NB)
        rate_sum += rate;
        active += rem ? 1u : 0u;
    }
    rate_sum = block_reduce<u64, NT>(rate_sum, sm.red, OpAdd());
    active = block_reduce<u32, NT>(active, (u32*)sm.red, OpAdd());
    const u64 spare = (u64)C::CAP - active;                   // P <= CAP / 4, so this is most of the slots
    u32 mine = 0;
    for (int p = p0; p < p1; ++p) {
        const uint4 ri = sm.rowinfo[p];
        const u32 rem = ri.z - ri.x;
        u32 n = rem;
        if (rem && !all_fit) {
            const u64 extra = rate_sum ? sm.hist2[p] * spare / rate_sum : 0;     // < 2^50 * 2^14: no overflow; the floors add up to <= spare
            n = 1u + (u32)extra;
            n = n < rem ? n : rem;
        }
        rown[p] = n;
        mine += n;
    }
    u32 total;
    u32 off = block_excl_scan<u32, NT>(mine, (u32*)sm.red, total);
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) marker[(wave * ITEMS + j) * WAVE + lane] = 0;
    __syncthreads();
    for (int p = p0; p < p1; ++p) {
        const u32 n = rown[p];
        sm.rowinfo[p].y = off;
        if (n) marker[off] = (unsigned short)(p + 1);
        off += n;
    }
    if (tid == 0) sm.rowinfo[P] = make_uint4(0u, total, 0u, 0u);
    __syncthreads();
    // the row of every slot: the latest marker at or before it.  Inside a wave's 64 * ITEMS slots by lane
    // moves; the marker that is open at the wave's first slot comes from the waves before it.
    u32 mk[ITEMS], nx[ITEMS];
    u32 run = 0;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const u32 slot = (u32)(wave * ITEMS + j) * WAVE + lane;
        mk[j] = marker[slot];
        nx[j] = slot + 1 < (u32)C::CAP ? marker[slot + 1] : 0u;
        u32 v = wave_scan(mk[j], OpMax());
        v = v > run ? v : run;
        run = (u32)__shfl((int)v, WAVE - 1, WAVE);
        slotrow[j] = v;                                       // for now: the latest marker inside the wave's range
    }
    u32* wmax = (u32*)sm.red;
    if (lane == 0) wmax[wave] = run;
    __syncthreads();
    u32 before = 0;
    for (int w = 0; w < wave; ++w) { const u32 x = wmax[w]; before = x > before ? x : before; }
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const u32 slot = (u32)(wave * ITEMS + j) * WAVE + lane;
        const u32 m = slotrow[j] > before ? slotrow[j] : before;
        u32 r = (u32)P;                                       // slots beyond the plan: the entry that is never active
        if (slot < total && m) {
            r = m - 1u;
            if (mk[j]) r |= SLOT_FIRST;
            if (slot + 1 == total || nx[j]) r |= SLOT_LAST;
        }
        slotrow[j] = r;
    }
    __syncthreads();                                          // the markers lie over the bucket words: done with them
    return total;
}

// The value as the compiler cannot see through it: keeps it from forming, once and for all steps, every
// (first slot + 64 * item) in a register of its own.
__device__ __forceinline__ u32 opaque(u32 x)
{
    asm volatile("" : "+v"(x));
    return x;
}

// The cursors move behind the consumed entries (key != KEY_NONE): the lane that holds a row's last consumed
// entry writes the row's new cursor.  Whether the slot after a wave's last one is consumed is read from
// misc[M_CARRY + wave + 1], which the next wave wrote before the last barrier.
template <int NT, int ITEMS>
__device__ __forceinline__ void sweep_move_cursors(const SweepSm& sm, const u32 (&key)[ITEMS], const u32 (&slotrow)[ITEMS], u32 slot0)
{
    constexpr int NW = NT / WAVE;
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x >> 6;
    u64 m = __ballot(key[0] != KEY_NONE);
    const u32 sg = opaque(slot0);
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        u64 mn;
        if (j + 1 < ITEMS) mn = __ballot(key[j + 1 < ITEMS ? j + 1 : j] != KEY_NONE);
        else mn = wave + 1 < NW ? (u64)sm.misc[M_CARRY + wave + 1] : 0ull;
        const u64 next = (m >> 1) | (mn << 63);
        const u64 lastm = __ballot((slotrow[j] & SLOT_LAST) != 0);
        const u64 E = m & (lastm | ~next);
        if ((E >> lane) & 1ull) {
            uint4* rp = sm.rowinfo + (slotrow[j] & SLOT_ROW);
            const uint2 r2 = *(const uint2*)rp;
            rp->x = (r2.x - r2.y + sg) + ((u32)j * WAVE + 1u);
        }
        m = mn;
    }
}

// One workgroup per slice of an instance; the slice's best candidate goes to partial[b * nslices + s].
template <int NT, int ITEMS, int PMAX>       // PMAX: the most rows the workgroup's LDS is laid out for
__global__ __launch_bounds__(NT, 4) void zl_sweep_kernel(
    const i64* __restrict__ ts, i64 B, int P, int R, int nslices,
    const InstInfo* __restrict__ info, const SegEntry* __restrict__ segtab,
    Partial* __restrict__ partial, int* __restrict__ status)
{
    using C = SweepCfg<NT, ITEMS>;
    constexpr int NW = C::NW;
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
    // the slice: values (relative to base) in [vs, ve)
    if (tid < 2) {
        const u32 k = s + (u32)tid;
        sm.red[tid] = k < ii.nb ? fine_bin_start(k, ii, segtab + b * (i64)SEGS) : ii.range + 1;
    }
    __syncthreads();
    const bool first_slice = s == 0, last_slice = s + 1 == ii.nb;
    const u64 vs = first_slice ? 0ull : sm.red[0], ve = last_slice ? ii.range + 1 : sm.red[1];
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
        W0 = block_reduce<u64, NT>(w0, sm.red, OpAdd());
        remaining = block_reduce<u32, NT>(rem, (u32*)sm.red, OpAdd());
        bad = __syncthreads_or(wrong);
    }
    if (tid == 0) { sm.misc[M_LIVE] = 0; sm.misc[M_OFFEND] = 0xffffffffu; sm.misc[M_FLAGS] = 0; sm.misc[M_STALE] = 0; }

    u64 A = vs;                                   // first value of the window to come (relative to base)
    const u64 thr = ii.thr;
    const u64 PP = (u64)(u32)P;
    i64 UB = INT64_MAX;                           // best upper bound of the minimum so far
    u64 best_w = U64_MAX, best_c = U64_MAX;       // this thread's best candidate: wait, barrier relative to base
    u32 slotrow[ITEMS];
    u32 key[ITEMS], dl[ITEMS];
    bool replan = true;
    const u32 slot0 = (u32)(wave * ITEMS) * WAVE + lane;
    const u64 step_cap = 2ull * remaining + 64;   // sorted rows never come near it
    const int chunk = (P + NT - 1) / NT;
    const int rp0 = tid * chunk, rp1 = rp0 + chunk < P ? rp0 + chunk : P;
    constexpr u64 SMASK = (1ull << 46) - 1;       // low field of a bucket word

    for (u64 step = 0; remaining > 0 && !bad; ++step) {
        if (step > step_cap) { bad = 1; break; }
        if (replan) {
            sweep_plan<NT, ITEMS>(sm, inst, P, base + A, remaining, slotrow);
            replan = false;
        }
        const u64 a_abs = base + A;
        // ---- the frontier: last loaded value of every row whose run does not reach the end of its entries
        // (as F + 1: 0 says that some such row's run ends before A, with entries equal to the last frontier
        // that were not loaded when it passed: then nothing but such entries can be passed over in this step)
        u32 fmin = SWEEP_SPAN_MAX + 1u;
        for (int p = rp0; p < rp1; ++p) {
            const uint4 ri = sm.rowinfo[p];
            const u32 n = sm.rowinfo[p + 1].y - ri.y;
            if (n && ri.x + n < ri.z) {
                const u64 rel = (u64)inst[ri.x + n - 1] - a_abs;
                const u32 f = (i64)rel < 0 ? 0u : ((rel >> 32) == 0 && (u32)rel < SWEEP_SPAN_MAX ? (u32)rel + 1u : SWEEP_SPAN_MAX + 1u);
                fmin = f < fmin ? f : fmin;
            }
        }
        // ---- clear the bucket words (everything of the step before has been read: barrier at its end)
        {
            uint4* h4 = (uint4*)(sm.hist + (size_t)tid * C::BPT);
            h4[0] = make_uint4(0u, 0u, 0u, 0u);
            h4[1] = make_uint4(0u, 0u, 0u, 0u);
        }
        // ---- zl_delta: the runs into (key, delta) records
        u32 gmask = 0, negacc = 0;
        constexpr int BATCH = ITEMS < 8 ? ITEMS : 8;
#pragma unroll
        for (int g = 0; g < ITEMS; g += BATCH) {
            i64 cur[BATCH], prd[BATCH];
            bool act[BATCH], head[BATCH];
            const u32 sg = opaque(slot0 + (u32)g * WAVE);
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {
                const uint4 ri = sm.rowinfo[slotrow[g + j] & SLOT_ROW];
                const u32 e = (ri.x - ri.y + sg) + (u32)j * WAVE;
                act[j] = e < ri.z;
                head[j] = e <= ri.w;                                      // the row's entry 0: its predecessor is base
                const u32 ce = act[j] ? e : 0u;
                const u32 pe = act[j] && !head[j] ? e - 1u : ce;
                cur[j] = inst[ce];
                prd[j] = inst[pe];
            }
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {
                const u64 c = (u64)cur[j];
                const u64 pr = act[j] && head[j] ? base : (u64)prd[j];
                const u64 rel = c - a_abs, d = c - pr;
                const bool okc = act[j] && (rel >> 32) == 0 && (u32)rel <= SWEEP_SPAN_MAX;
                u32 k = okc ? (u32)rel : KEY_NONE;
                const bool stale = act[j] && (i64)rel < 0;                // before A: in sorted rows a repeat of the last frontier
                if (stale) k = KEY_STALE;
                key[g + j] = k;
                dl[g + j] = (u32)d;
                const u32 an = (u32)(d >> 32) | ((u32)d >> 31);           // a step of 2^31 or more, or backwards
                gmask |= an ? 1u << (g + j) : 0u;
                negacc |= (u32)(d >> 32) | (stale && d != 0 ? 0x80000000u : 0u);
            }
        }
        fmin = wave_scan(fmin, OpMin());
        if (lane == WAVE - 1) ((u32*)sm.red)[wave] = fmin;
        {
            u32 fl = (negacc >> 31) ? FLAG_NEG : 0u;
            fl |= gmask ? FLAG_GIANT : 0u;
            if (fl) atomicOr(&sm.misc[M_FLAGS], fl);
        }
        __syncthreads();                                                  // B1
        u32 F1 = ((u32*)sm.red)[0];
#pragma unroll
        for (int w = 1; w < NW; ++w) { const u32 x = ((u32*)sm.red)[w]; F1 = x < F1 ? x : F1; }
        const u32 flags = sm.misc[M_FLAGS];
        if (flags & FLAG_NEG) { bad = 1; break; }
        if (F1 == 0) {
            // only repeats of the last frontier are passed over: the cursors move, A and W0 stay
            u32 nstale = 0;
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                if (key[j] != KEY_STALE) key[j] = KEY_NONE;
                nstale += (u32)__popcll(__ballot(key[j] == KEY_STALE));
            }
            if (lane == 0) {
                sm.misc[M_CARRY + wave] = key[0] != KEY_NONE ? 1u : 0u;
                if (nstale) atomicAdd(&sm.misc[M_STALE], nstale);
            }
            __syncthreads();
            const u32 stale = sm.misc[M_STALE];
            if (stale == 0) { bad = 1; break; }                          // (sorted rows always have such entries here)
            sweep_move_cursors<NT, ITEMS>(sm, key, slotrow, slot0);
            remaining -= stale < remaining ? stale : remaining;
            __syncthreads();
            if (tid == 0) { sm.misc[M_LIVE] = 0; sm.misc[M_OFFEND] = 0xffffffffu; sm.misc[M_FLAGS] = 0; sm.misc[M_STALE] = 0; }
            __syncthreads();
            continue;
        }
        u32 F = F1 - 1u;
        if (ve - 1 - A < (u64)F) F = (u32)(ve - 1 - A);                   // the slice ends there: no entry of it lies beyond
        const bool anyg = (flags & FLAG_GIANT) != 0;
        if (anyg) {
            uint4* g4 = (uint4*)(sm.hist2 + (size_t)tid * C::BPT);
            g4[0] = make_uint4(0u, 0u, 0u, 0u);
            g4[1] = make_uint4(0u, 0u, 0u, 0u);
            __syncthreads();
        }
        const u64 need64 = thr > A ? thr - A : 0ull;
        const u32 need = need64 > 0xffffffffull ? 0xffffffffu : (u32)need64;      // keys >= need are admissible

        // ---- consume the window [A, A + F]; taken again with a smaller F if the buckets cannot be evaluated
        u32 sh, consumed = 0, stale = 0, live = 0;
        u64 dsum = 0;
        for (;;) {
            sh = bit_length((u64)F) > C::LOG_NB ? (u32)(bit_length((u64)F) - C::LOG_NB) : 0u;
            u32 nstale = 0;
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                u32 k = key[j];
                if (k > F && k != KEY_STALE) k = KEY_NONE;
                key[j] = k;
                if (k <= F) {
                    const bool giant = (gmask >> j) & 1u;
                    atomicAdd(&sm.hist[k >> sh], (1ull << 46) | (giant ? 0ull : (u64)dl[j]));
                }
                nstale += (u32)__popcll(__ballot(k == KEY_STALE));
            }
            if (anyg) {          // the deltas of 2^31 or more: formed again from the entries themselves
                const u32 sg = opaque(slot0);
#pragma unroll
                for (int j = 0; j < ITEMS; ++j)
                    if (((gmask >> j) & 1u) && key[j] <= F) {
                        const uint4 ri = sm.rowinfo[slotrow[j] & SLOT_ROW];
                        const u32 e = (ri.x - ri.y + sg) + (u32)j * WAVE;
                        const u64 pr = e <= ri.w ? base : (u64)inst[e - 1];
                        if (e < ri.z) atomicAdd(&sm.hist2[key[j] >> sh], (u64)inst[e] - pr);
                    }
            }
            if (lane == 0) {
                sm.misc[M_CARRY + wave] = key[0] != KEY_NONE ? 1u : 0u;       // is the wave's first slot consumed
                if (nstale) atomicAdd(&sm.misc[M_STALE], nstale);
            }
            __syncthreads();                                              // B2
            // ---- zl_scan over the buckets, four per thread; bounds; which buckets survive
            u64 h[C::BPT], gg[C::BPT];
            {
                const uint4* h4 = (const uint4*)(sm.hist + (size_t)tid * C::BPT);
                const uint4 a0 = h4[0], a1 = h4[1];
                h[0] = (u64)a0.x | ((u64)a0.y << 32); h[1] = (u64)a0.z | ((u64)a0.w << 32);
                h[2] = (u64)a1.x | ((u64)a1.y << 32); h[3] = (u64)a1.z | ((u64)a1.w << 32);
            }
            gg[0] = gg[1] = gg[2] = gg[3] = 0;
            if (anyg) {
#pragma unroll
                for (int i = 0; i < C::BPT; ++i) gg[i] = sm.hist2[tid * C::BPT + i];
            }
            const u64 tot = h[0] + h[1] + h[2] + h[3];
            const u64 gtot = gg[0] + gg[1] + gg[2] + gg[3];
            const u64 inc = wave_scan(tot, OpAdd());
            const u64 ginc = anyg ? wave_scan(gtot, OpAdd()) : 0ull;
            u32 lo[C::BPT], hi[C::BPT];
#pragma unroll
            for (int i = 0; i < C::BPT; ++i) {
                lo[i] = (u32)(tid * C::BPT + i) << sh;
                const u32 top = lo[i] + ((1u << sh) - 1u);
                hi[i] = top < F ? top : F;
            }
            // smallest P*hi - E over the admissible buckets, E counted from the wave's first bucket
            i64 u = INT64_MAX;
            {
                u64 e = (inc - tot) & SMASK, ge = ginc - gtot;
#pragma unroll
                for (int i = 0; i < C::BPT; ++i) {
                    e += h[i] & SMASK;
                    ge += gg[i];
                    if ((h[i] >> 46) && lo[i] >= need) {
                        const i64 x = (i64)(PP * hi[i] - e - ge);
                        u = x < u ? x : u;
                    }
                }
            }
            u = wave_scan(u, OpMin());
            if (lane == WAVE - 1) { sm.red[wave] = inc; sm.red[NW + wave] = (u64)u; sm.red[2 * NW + wave] = ginc; }
            __syncthreads();                                              // Bs
            u64 hbase = 0, total = 0, gbase = 0, gsum = 0;
            i64 um = INT64_MAX;
#pragma unroll 2
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
            consumed = (u32)(total >> 46);
            dsum = (total & SMASK) + gsum;
            stale = sm.misc[M_STALE];
            i64 ubn = UB;
            if (um != INT64_MAX) { const i64 x = um + (i64)W0; ubn = x < ubn ? x : ubn; }
            const i64 ubrel = ubn == INT64_MAX ? ubn : ubn - (i64)W0;
            {
                u64 e = hbase & SMASK, ge = gbase;
                u32 at[C::BPT];
                u64 eb[C::BPT], gb[C::BPT];
#pragma unroll
                for (int i = 0; i < C::BPT; ++i) {
                    const u32 c = (u32)(h[i] >> 46);
                    eb[i] = e;
                    gb[i] = ge;
                    e += h[i] & SMASK;
                    ge += gg[i];
                    at[i] = SWEEP_DROPPED;
                    if (sh == 0) {
                        // a bucket is one value: its prefix sum is the candidate's
                        if (c && lo[i] >= need) {
                            const u64 w = PP * lo[i] + W0 - e - ge;
                            const u64 cabs = A + lo[i];
                            if (w < best_w || (w == best_w && cabs < best_c)) { best_w = w; best_c = cabs; }
                        }
                    } else if (c && hi[i] >= need && (i64)(PP * lo[i] - e - ge) <= ubrel) {
                        if (c > SWEEP_DEEP || gg[i]) atomicMin(&sm.misc[M_OFFEND], (u32)(tid * C::BPT + i));
                        at[i] = atomicAdd(&sm.misc[M_LIVE], c);
                    }
                }
                if (sh != 0) {
#pragma unroll
                    for (int i = 0; i < C::BPT; ++i) {
                        sm.cnt[tid * C::BPT + i] = at[i];
                        sm.hist[tid * C::BPT + i] = eb[i] | ((u64)(at[i] & 0x3ffffu) << 46);
                        if (anyg) sm.hist2[tid * C::BPT + i] = gb[i];
                    }
                }
            }
            __syncthreads();                                              // B3
            if (sh == 0) { UB = ubn; break; }
            live = sm.misc[M_LIVE];
            const u32 off = sm.misc[M_OFFEND];
            if (off == 0xffffffffu && live <= (u32)C::LIST) { UB = ubn; break; }
            // not to be evaluated entry by entry: up to the offending bucket, or (if it is the first) that bucket alone, cut finer
            u32 fnew = off == 0xffffffffu ? F >> 1 : (off > 0 ? (off << sh) - 1u : (1u << sh) - 1u);
            if (fnew >= F) fnew = F >> 1;
            F = fnew;
            __syncthreads();                                              // everyone has read the step's words
            if (tid == 0) { sm.misc[M_LIVE] = 0; sm.misc[M_OFFEND] = 0xffffffffu; sm.misc[M_STALE] = 0; }
            {
                uint4* h4 = (uint4*)(sm.hist + (size_t)tid * C::BPT);
                h4[0] = make_uint4(0u, 0u, 0u, 0u);
                h4[1] = make_uint4(0u, 0u, 0u, 0u);
                if (anyg) {
                    uint4* g4 = (uint4*)(sm.hist2 + (size_t)tid * C::BPT);
                    g4[0] = make_uint4(0u, 0u, 0u, 0u);
                    g4[1] = make_uint4(0u, 0u, 0u, 0u);
                }
            }
            __syncthreads();
        }

        if (consumed + stale == 0) {
            // nothing at or below F (a gap wider than a window): go to the smallest loaded value
            u64 amin = U64_MAX;
            const u32 sg = opaque(slot0);
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                const uint4 ri = sm.rowinfo[slotrow[j] & SLOT_ROW];
                const u32 e = (ri.x - ri.y + sg) + (u32)j * WAVE;
                if (e < ri.z) {
                    const u64 rel = (u64)inst[e] - base;
                    amin = rel < amin ? rel : amin;
                }
            }
            amin = block_reduce<u64, NT>(amin, sm.red, OpMin());
            if (amin == U64_MAX || amin <= A + F) { bad = 1; break; }        // only rows that are not sorted get here
            W0 += PP * (amin - A);
            A = amin;
            if (tid == 0) { sm.misc[M_LIVE] = 0; sm.misc[M_OFFEND] = 0xffffffffu; sm.misc[M_FLAGS] = 0; sm.misc[M_STALE] = 0; }
            __syncthreads();
            continue;
        }

        sweep_move_cursors<NT, ITEMS>(sm, key, slotrow, slot0);
        // ---- zl_argmin over the entries of the surviving buckets
        if (sh != 0 && live > 0) {
#pragma unroll
            for (int j = 0; j < ITEMS; ++j)
                if (key[j] <= F) {
                    const u32 bq = key[j] >> sh;
                    if (sm.cnt[bq] < SWEEP_DROPPED) {
                        const u32 slot = atomicAdd(&sm.cnt[bq], 1u);
                        if (slot < (u32)C::LIST) sm.recs[slot] = (u64)key[j] | ((u64)dl[j] << 32);
                    }
                }
            __syncthreads();                                              // B4
            for (u32 q = tid; q < live; q += NT) {
                const u32 k = (u32)sm.recs[q];
                const u32 bq = k >> sh;
                const u32 e = sm.cnt[bq];
                const u64 hb = sm.hist[bq];
                u32 x = (u32)(hb >> 46);
                u64 S = hb & SMASK;
                if (anyg) S += sm.hist2[bq];
                for (; x < e; ++x) {
                    const u64 r = sm.recs[x];
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
        remaining -= consumed + stale;
        // a new plan where the runs have grown uneven (rows ending, speeds changing), and for the last entries
        if (remaining > 0 && (2 * (consumed + stale) < (u32)C::CAP)) replan = true;
        if (tid == 0) { sm.misc[M_LIVE] = 0; sm.misc[M_OFFEND] = 0xffffffffu; sm.misc[M_FLAGS] = 0; sm.misc[M_STALE] = 0; }
        __syncthreads();                                                  // end of the step
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

// The fast search of one window: value buckets, exact bounds, evaluation of the surviving entries.
// Part of the ZipLine library (see zipline.hip); device code for gfx950.
#pragma once
#include "zl_sort.h"

namespace {

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

// The records of a window, held ITEMS per thread in registers (item j of thread t
// is record j*NT + t, present if that is below `total`) -> first minimum
// (wait, key) of P*key + W0 - S(key) over keys with a + key >= thr, W0 being the
// block sum of `w0` (taken as 0 unless WITH_W0).
// On entry the bucket words must be zero and a barrier must have passed since;
// the record area may hold anything (it is overwritten).  On return some threads
// may still be reading LDS: the caller passes a barrier before writing it again.
// Returns false (nothing computed) if some bucket is over the limit.
//
// Which of a thread's items exist is the caller's to say: Present::operator()(j).  The default
// is the strided layout above (SlotsBelow).  LIST_CAP > 0: the record area holds only that many
// records (at least 2 * BUCKET_LIMIT); if more entries survive the bounds they are scattered and
// evaluated in rounds, whole buckets at a time (only with a map that has bounds).
template <int NT>
struct SlotsBelow {           // item j of thread t is slot j*NT + t of `total`
    int total;
    __device__ __forceinline__ bool operator()(int j) const { return j * NT + (int)threadIdx.x < total; }
};
// The deltas are the caller's too: Delta::operator()(j), called by all threads together for every
// j (also for items that do not exist), so that it may take its value from a neighbouring lane.
template <int ITEMS>
struct StoredDeltas {         // the deltas sit in registers
    const u32 (&dl)[ITEMS];
    __device__ __forceinline__ u32 operator()(int j) const { return dl[j]; }
};
template <int NT, int ITEMS, bool WITH_W0, class Map, int LIST_CAP = 0, class Present = SlotsBelow<NT>,
          class Delta = StoredDeltas<ITEMS>>
__device__ __forceinline__ bool zl_bucket_finish(const Smem& sm, const u32 (&key)[ITEMS], const Delta delta,
                                                 const Map bucket, const Present present, u64 a, u64 thr, u32 P, u64 w0,
                                                 u64& best_wait, u32& best_key)
{
    using H = HotCfg<NT, ITEMS>;
    static_assert(LIST_CAP == 0 || (Map::HAS_BOUNDS && LIST_CAP >= 2 * (int)BUCKET_LIMIT), "a short list needs the bounds");
    u64* recs = sm.recs;
    u64* bsum = sm.red - H::NB;                                       // the bucket words end where the scratch begins
    u32* cnt = sm.cnt;
    const int tid = threadIdx.x;
    u32* live_count = (u32*)(sm.red + H::RED_WORDS - 1);              // entries of the compact list
    u32* deep = live_count + 1;                                       // set if some bucket is over the limit
    if (tid == 0) { *live_count = 0; *deep = 0; }
    // zl_sort, step 1: per bucket, entry count and sum of deltas in one word
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const u32 d = delta(j);
        if (present(j)) {
            const u32 bid = bucket(key[j]);
            atomicAdd(&bsum[bid], (1ull << SUM_BITS) | (u64)d);
        }
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
        // BP(bucket) and the bucket's first slot (all ones in that field: the bucket is dropped)
        constexpr u32 FIRST_MASK = (1u << (64 - SUM_BITS)) - 1u;
        bsum[2 * tid] = sbase | ((u64)(live0 ? at0 : (LIST_CAP ? FIRST_MASK : 0u)) << SUM_BITS);
        bsum[2 * tid + 1] = e0 | ((u64)(live1 ? at1 : (LIST_CAP ? FIRST_MASK : 0u)) << SUM_BITS);
        __syncthreads();
        const int live = (int)*live_count;
        auto evaluate = [&](u32 k, u32 x, u32 e, u64 S) {           // candidate k: its bucket's records are [x, e)
            for (; x < e; ++x) {
                const u64 r = recs[x];
                S += ((u32)r <= k) ? r >> 32 : 0ull;
            }
            if ((u64)k >= need) {
                const u64 w = (u64)P * k + W0 - S;
                if (w < bw || (w == bw && k < bk)) { bw = w; bk = k; }
            }
        };
        if (LIST_CAP == 0 || live <= LIST_CAP) {
            // step 3: scatter the entries of the live buckets; afterwards cnt[b] is the end of bucket b
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
                const u32 d = delta(j);
                if (present(j)) {
                    const u32 bid = bucket(key[j]);
                    const u32 slot = atomicAdd(&cnt[bid], 1u);
                    if (slot < DROPPED) recs[slot] = (u64)key[j] | ((u64)d << 32);
                }
            }
            __syncthreads();
            // zl_scan + zl_argmin: every listed entry evaluates its own candidate
            for (int q = tid; q < live; q += NT) {
                const u32 k = (u32)recs[q];
                const u32 bid = bucket(k);
                const u64 hb = bsum[bid];
                evaluate(k, (u32)(hb >> SUM_BITS), cnt[bid], hb & SUM_MASK);
            }
        } else {
            // More survivors than the list holds: rounds of whole buckets.  A bucket belongs to the round
            // its first slot falls in; it has at most BUCKET_LIMIT entries, so a round's slots, counted
            // from the round's start, stay below LIST_CAP.
            constexpr u32 ROUND = (u32)LIST_CAP - BUCKET_LIMIT;
            for (u32 r0 = 0; r0 < (u32)live; r0 += ROUND) {
#pragma unroll
                for (int j = 0; j < ITEMS; ++j) {
                    const u32 d = delta(j);
                    if (present(j)) {
                        const u32 bid = bucket(key[j]);
                        const u32 first = (u32)(bsum[bid] >> SUM_BITS);
                        if (first >= r0 && first - r0 < ROUND) {
                            const u32 slot = atomicAdd(&cnt[bid], 1u);
                            recs[slot - r0] = (u64)key[j] | ((u64)d << 32);
                        }
                    }
                }
                __syncthreads();
                const u32 span = (u32)live - r0 < (u32)LIST_CAP ? (u32)live - r0 : (u32)LIST_CAP;
                for (u32 q = tid; q < span; q += NT) {
                    // a slot of this round holds a record iff it lies inside its own bucket's slots and
                    // that bucket belongs to the round (anything else is left over from earlier)
                    const u32 k = (u32)recs[q];
                    const u32 bid = bucket(k);
                    const u64 hb = bsum[bid];
                    const u32 first = (u32)(hb >> SUM_BITS), e = cnt[bid];
                    if (first >= r0 && first - r0 < ROUND && q + r0 >= first && q + r0 < e)
                        evaluate(k, first - r0, e - r0, hb & SUM_MASK);
                }
                __syncthreads();
            }
        }
    } else {
    cnt[2 * tid] = cbase; cnt[2 * tid + 1] = cbase + c0;
    bsum[2 * tid] = sbase | ((u64)cbase << SUM_BITS);                 // BP(bucket) and the bucket's first slot
    bsum[2 * tid + 1] = (sbase + s0) | ((u64)(cbase + c0) << SUM_BITS);
    __syncthreads();
    // step 3: scatter; afterwards cnt[b] is the end of bucket b
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const u32 d = delta(j);
        if (present(j)) {
            const u32 bid = bucket(key[j]);
            const u32 slot = atomicAdd(&cnt[bid], 1u);
            recs[slot] = (u64)key[j] | ((u64)d << 32);
        }
    }
    // a 4-wide read of the last bucket may run past the end: entries that add nothing
    const int total = present.total;              // (this form is for the strided layout)
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

}  // namespace

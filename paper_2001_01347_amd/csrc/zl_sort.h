// The general search of one window workgroup: LDS layout, radix sort, prefix scan, arg-min.
// Part of the ZipLine library (see zipline.hip); device code for gfx950.
#pragma once
#include "zl_rows.h"

namespace {

// Window workgroup: LDS layout and the sort/scan/argmin steps.
//
// A record is (key: low 32 bits, delta: high 32 bits).  Keys are relative to
// the window start and windows are at most 2^32 wide.  Deltas fit 32 bits when
// the instance's range does; otherwise (WIDE) the upper half of each delta
// lives in a second plane and a window holds half as many records (a third
// plane of the same size carries one more payload word for the searches that
// need it).  Record q
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
    static constexpr size_t REC_BYTES = (size_t)RECS * 8 > (size_t)RECS_WIDE * 16 ? (size_t)RECS * 8 : (size_t)RECS_WIDE * 16;
    static constexpr int CNT_WORDS = (NW * RADIX_MAX > 2 * NT) ? NW * RADIX_MAX : 2 * NT;
    static constexpr int RED_WORDS = 3 * NW + 8;          // u64 scratch for scans and reductions
    static constexpr size_t BYTES = (REC_BYTES + 15) / 16 * 16 + (size_t)RED_WORDS * 8 + (size_t)CNT_WORDS * 4;
};

struct Smem {       // carved from one static LDS array
    u64* recs;      // record plane
    u32* dhi;       // upper halves of the deltas (WIDE only)
    u32* ext;       // one more payload word per record (WIDE with EXTRA only)
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
    s.ext = s.dhi + C::RECS_WIDE;
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
// KEYHI: the third plane holds the upper halves of 64-bit keys and takes part in the order
// (kbits up to 64); otherwise it is payload.
template <int NT, int ITEMS, bool WIDE, bool EXTRA = false, bool KEYHI = false>
__device__ __forceinline__ void zl_sort(const Smem& sm, int items, int kbits)
{
    static_assert(WIDE || !EXTRA, "the third plane goes with the WIDE layout");
    static_assert(EXTRA || !KEYHI, "upper key halves live in the third plane");
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
        u32 key[IT], dl[IT], dh[WIDE ? IT : 1], ex[EXTRA ? IT : 1], rank[IT];
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            if (j < items) {
                const u64 r = recs[phys(wbase + j * WAVE)];
                key[j] = (u32)r;
                dl[j] = (u32)(r >> 32);
                if (WIDE) dh[j] = sm.dhi[phys(wbase + j * WAVE)];
                if (EXTRA) ex[j] = sm.ext[phys(wbase + j * WAVE)];
                const u32 d = KEYHI ? (u32)(((u64)key[j] | ((u64)ex[j] << 32)) >> sh) & dmask : (key[j] >> sh) & dmask;
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
                const u32 d = KEYHI ? (u32)(((u64)key[j] | ((u64)ex[j] << 32)) >> sh) & dmask : (key[j] >> sh) & dmask;
                const int pos = (int)(mycnt[d] + rank[j]);
                recs[phys(pos)] = (u64)key[j] | ((u64)dl[j] << 32);
                if (WIDE) sm.dhi[phys(pos)] = dh[j];
                if (EXTRA) sm.ext[phys(pos)] = ex[j];
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
// KEY64: keys are 64 bits wide, their upper halves in the third plane.
template <int NT, bool WIDE, bool KEY64 = false>
__device__ __forceinline__ void zl_scan_argmin(const Smem& sm, int items, int total,
                                               u64 a, u64 thr, u64 P, u64 W0,
                                               u64& best_wait, u64& best_key)
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
    u32 bq = 0xffffffffu;
    u64 bk = 0;
    u64 r = (q0 < qe) ? recs[phys(q0)] : 0ull;
    u32 rh = (KEY64 && q0 < qe) ? sm.ext[phys(q0)] : 0u;
    for (int q = q0; q < qe; ++q) {
        const u64 key = (u64)(u32)r | ((u64)rh << 32);
        S += r >> 32;
        if (WIDE) S += (u64)sm.dhi[phys(q)] << 32;
        const bool has_next = q + 1 < total;
        const u64 rn = has_next ? recs[phys(q + 1)] : 0ull;
        const u32 rnh = (KEY64 && has_next) ? sm.ext[phys(q + 1)] : 0u;
        const bool run_end = !has_next || ((u64)(u32)rn | ((u64)rnh << 32)) != key;
        const bool admissible = a + key >= thr;
        if (run_end && admissible) {
            const u64 w = P * key + W0 - S;
            if (w < bw) { bw = w; bq = (u32)q; bk = key; }
        }
        r = rn;
        rh = rnh;
    }
    // block arg-min over (wait, position): smaller wait, then earlier position
#pragma unroll
    for (int d = WAVE / 2; d > 0; d >>= 1) {
        const u64 ow = __shfl_xor(bw, d, WAVE);
        const u32 oq = __shfl_xor(bq, d, WAVE);
        const u64 ok = __shfl_xor(bk, d, WAVE);
        if (ow < bw || (ow == bw && oq < bq)) { bw = ow; bq = oq; bk = ok; }
    }
    constexpr int NW = NT / WAVE;
    const int lane = tid & (WAVE - 1), wave = tid >> 6;
    if (lane == 0) { red[wave] = bw; red[NW + wave] = bq; red[2 * NW + wave] = bk; }
    __syncthreads();
    bw = red[0];
    bq = (u32)red[NW];
    bk = red[2 * NW];
#pragma unroll
    for (int w = 1; w < NW; ++w) {
        const u64 ow = red[w];
        const u32 oq = (u32)red[NW + w];
        if (ow < bw || (ow == bw && oq < bq)) { bw = ow; bq = oq; bk = red[2 * NW + w]; }
    }
    __syncthreads();
    best_wait = bw;
    best_key = bk;
}

// Sentinels behind the last record, so that whole rounds of 64 can be sorted.
template <int NT>
__device__ __forceinline__ void fill_sentinels(u64* recs, int total, int items)
{
    for (int q = total + threadIdx.x; q < NT * items; q += NT) recs[phys(q)] = 0x00000000ffffffffull;
}

// The same for the plane of upper key halves.
template <int NT>
__device__ __forceinline__ void fill_sentinels_hi(u32* ext, int total, int items)
{
    for (int q = total + threadIdx.x; q < NT * items; q += NT) ext[phys(q)] = 0xffffffffu;
}

// zl_delta for a value interval [a, el] (el - a < 2^32, or any width with KEY64: the upper
// halves of the keys then go to the third plane) of the rows in `rw`:
// gathers every row's segment into records (key = value - a, delta = value -
// the row's previous value, or value - a for a row's very first entry) in
// slots [0, total).  At most `cap` records are stored; the true total is
// returned.  w0 accumulates this thread's share of W0 = sum_p (a - last value
// of row p before the interval).  Rows are taken NT at a time: a block scan of
// the segment lengths gives every row its first slot, then consecutive threads
// take consecutive slots, so reads within a segment coalesce.
template <int NT, bool WIDE, bool PAD, bool KEY64 = false>
__device__ __forceinline__ int zl_delta(const Smem& sm, const Rows& rw, u64 a, u64 el, bool lx, bool rx,
                                        int cap, u64& w0, int& bad)
{
    static_assert(WIDE || !KEY64, "64-bit keys go with the three-plane layout");
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
            if (KEY64) sm.ext[slot] = (u32)((rel - a) >> 32);
        }
        total += (int)chunk;
        __syncthreads();
    }
    return total;
}

}  // namespace

// One workgroup per instance: the whole search in LDS.
// Part of the ZipLine library (see zipline.hip); device code for gfx950.
#pragma once
#include "zl_walk.h"

namespace {

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
                u64 tw, iw;
                table_entry(below_c, c[i], (u32)n, (u32)H::NB, bucket.cshift, tw, iw);
                tab[tid * CPT + i] = tw;
                tab[H::COARSE + tid * CPT + i] = iw;
            }
            below_c += c[i];
        }
    }
    __syncthreads();
    u64 best_wait;
    u32 bkey;
    if (!zl_bucket_finish<NT, ITEMS, false>(sm, key, StoredDeltas<ITEMS>{dl}, bucket, SlotsBelow<NT>{n}, 0ull, thr, (u32)P, 0ull, best_wait, bkey)) {
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

// The same search for the larger single-workgroup instances (1024 < P*R <= NT*ITEMS) with the
// keys held in registers from the loads to the evaluation: LDS holds only the bucket words,
// the tables and a short list of the entries that survive the bounds, so that several
// workgroups share a CU and one loads while another searches.  The instance's bounds come first,
// from the ends of its rows, and stay in scalar registers; the keys are relative to base from
// the start.  Wave w holds elements [w*64*items, (w+1)*64*items), 64 consecutive ones per item,
// so an element's predecessor sits in the neighbouring lane and its delta is never stored.
template <int NT, int ITEMS>
struct WaveItems {            // which of a thread's items exist in that layout
    u32 mask;
    __device__ __forceinline__ bool operator()(int j) const { return (mask >> j) & 1u; }
};
template <int ITEMS>
struct NeighbourDeltas {      // an entry's delta is its key minus the key in the lane before, a row's first entry's its key
    const u32 (&key)[ITEMS];
    u32 heads;                // items that are a row's first entry
    u32 ahead;                // key of the element before the wave's first
    __device__ __forceinline__ u32 operator()(int j) const
    {
        u32 pk = dpp_take<DPP_WAVE_SHR1, 0xf>(0u, key[j]);
        const u32 edge = j > 0 ? last_lane(key[j > 0 ? j - 1 : 0]) : ahead;
        if ((threadIdx.x & (WAVE - 1)) == 0) pk = edge;
        return ((heads >> j) & 1u) ? key[j] : key[j] - pk;
    }
};
template <int NT, int ITEMS>
struct RegCfg {
    using H = HotCfg<NT, ITEMS>;
    static constexpr int LIST = NT >= 1024 ? 6144 : NT * ITEMS / 2;   // records of the short list: two, three or six workgroups fit a CU
    static constexpr size_t BYTES = (size_t)LIST * 8 + (size_t)H::NB * 8 + (size_t)H::RED_WORDS * 8 + (size_t)H::NB * 4 +
                                    (size_t)H::COARSE * 16;
};
template <int NT, int ITEMS, bool PRED>
__global__ __launch_bounds__(NT, (NT == 1024 ? 8 : (NT == 128 ? 5 : 6))) void zl_instance_reg_kernel(
    const i64* __restrict__ ts, const i64* __restrict__ le, const i64* __restrict__ iv, int P, int R, int rshift,
    i64* __restrict__ barrier, int* __restrict__ iters, i64* __restrict__ wait,
    int* __restrict__ status)
{
    using H = HotCfg<NT, ITEMS>;
    using C = RegCfg<NT, ITEMS>;
    static_assert(ITEMS <= 32 && ITEMS % 8 == 0, "item masks are one word; loads go in batches of 8");
    __shared__ __align__(16) unsigned char smem[C::BYTES];
    Smem sm;
    sm.recs = (u64*)smem;                                  // the short list
    sm.dhi = nullptr;
    sm.red = sm.recs + C::LIST + H::NB;                    // the bucket words sit between the list and the scratch
    sm.cnt = (u32*)(sm.red + H::RED_WORDS);                // followed by the coarse tables

    const int tid = threadIdx.x;
    const i64 b = blockIdx.x;
    const int n = P * R;
    const i64* __restrict__ inst = PRED ? nullptr : ts + b * (i64)n;
    const i64* __restrict__ lep = PRED ? le + b * (i64)P : nullptr;
    const i64* __restrict__ ivp = PRED ? iv + b * (i64)P : nullptr;
    // e / R for e < 2^16 (n <= 16384 here): exact with the rounded-up reciprocal, R >= 3 where it is used
    const u32 rinv = rshift >= 0 ? 0u : 0xffffffffu / (u32)R + 1u;
    auto row_of = [&](int e) -> int { return rshift >= 0 ? (e >> rshift) : (int)__umulhi((u32)e, rinv); };
    auto at = [&](int e) -> i64 {                          // element e of the instance
        if (!PRED) return inst[e];
        const int p = row_of(e);
        return (i64)((u64)lep[p] + (u64)(e - p * R + 1) * (u64)ivp[p]);
    };
    {
        u64* bsum = sm.red - H::NB;
        bsum[tid] = 0; bsum[tid + NT] = 0;
    }
    // the equalising bucket map needs the key counts of up to 256 coarse bins: counted while the records load
    u32* coarse = sm.cnt;                                   // free until the bucket scan
    u64* tab = (u64*)(sm.cnt + H::NB);
    constexpr int CPT = H::COARSE / NT > 1 ? H::COARSE / NT : 1;      // coarse bins per thread
    static_assert(H::NB >= H::COARSE, "the counters' area holds the coarse counts first");
#pragma unroll
    for (int i = 0; i < CPT; ++i)
        if (tid * CPT + i < H::COARSE) coarse[tid * CPT + i] = 0;
    // the instance's bounds from the ends of its rows (the exchange also orders the zeroes above)
    i64 base, first_max, last_max;
    {
        i64 mn = INT64_MAX, mxf = INT64_MIN, mxl = INT64_MIN;      // min first, max first, max last of the rows
        for (int p = tid; p < P; p += NT) {
            const i64 f = at(p * R), l = at(p * R + R - 1);
            mn = f < mn ? f : mn;
            mxf = f > mxf ? f : mxf;
            mxl = l > mxl ? l : mxl;
        }
        block_bounds<NT>(mn, mxf, mxl, (i64*)sm.red, base, first_max, last_max);
        base = (i64)uniform((u64)base);                    // the same in every thread: scalar registers
        first_max = (i64)uniform((u64)first_max);
        last_max = (i64)uniform((u64)last_max);
    }
    const u64 range = (u64)last_max - (u64)base;
    const u64 thr = (u64)first_max - (u64)base;
    u32 flags = 0;
    if (range > (u64)INT64_MAX / (u64)P) flags |= EBSP_STATUS_OVERFLOW;
    if (range >> 32) {
        // deltas need more than 32 bits: left to zl_instance_general_kernel
        if (tid == 0) wait[b] = DEFERRED;
        return;
    }
    const int bl = bit_length(range);
    TableMap<true> bucket;
    bucket.tab = tab;
    bucket.cshift = bl > 8 ? (u32)(bl - 8) : 0u;
    bucket.cmask = (1u << bucket.cshift) - 1u;
    bucket.span = (u32)range;

    const int lane = tid & (WAVE - 1), wave = tid >> 6;
    const int items = (n + NT - 1) / NT;
    const int wbase = wave * WAVE * items;
    i64 carry = (wbase > 0 && wbase < n) ? at(wbase - 1) : base;  // element ahead of the wave's first
    const u32 ahead = (u32)((u64)carry - (u64)base);               // its key
    int bad = 0;
    u32 key[ITEMS];                                        // relative to base
    u32 have = 0, heads = 0;                               // items that exist; items that are a row's first entry
    constexpr int LB = 8;                                  // loads of a thread in flight together
#pragma unroll
    for (int g = 0; g < ITEMS; g += LB) {
#pragma unroll
        for (int j = 0; j < LB; ++j) key[g + j] = 0;
        if (g < items) {
            i64 v[LB];
#pragma unroll
            for (int j = 0; j < LB; ++j) {
                const int e = wbase + (g + j) * WAVE + lane;
                v[j] = (g + j < items && e < n) ? at(e) : 0;
            }
#pragma unroll
            for (int j = 0; j < LB; ++j) {
                const int e = wbase + (g + j) * WAVE + lane;
                i64 prv = dpp_take<DPP_WAVE_SHR1, 0xf>((i64)0, v[j]);
                if (lane == 0) prv = carry;
                carry = (i64)last_lane((u64)v[j]);
                if (g + j < items && e < n) {
                    const bool first = e == row_of(e) * R;
                    const u32 rel = (u32)((u64)v[j] - (u64)base);   // (beyond the range only in unsorted rows: the maps clamp)
                    have |= 1u << (g + j);
                    key[g + j] = rel;
                    if (first) heads |= 1u << (g + j);
                    else bad |= (v[j] < prv);
                    atomicAdd(&coarse[bucket.coarse(rel)], 1u);
                }
            }
        }
    }
    const WaveItems<NT, ITEMS> present{have};
    if (__syncthreads_or(bad)) flags |= EBSP_STATUS_UNSORTED;       // also: the coarse counts are complete
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
                u64 tw, iw;
                table_entry(below_c, c[i], (u32)n, (u32)H::NB, bucket.cshift, tw, iw);
                tab[tid * CPT + i] = tw;
                tab[H::COARSE + tid * CPT + i] = iw;
            }
            below_c += c[i];
        }
    }
    __syncthreads();
    u64 best_wait;
    u32 bkey;
    // the deltas are not stored: an entry's delta is its key minus the key in the lane before (a row's first
    // delta is its key relative to base)
    const bool found = zl_bucket_finish<NT, ITEMS, false, TableMap<true>, C::LIST, WaveItems<NT, ITEMS>, NeighbourDeltas<ITEMS>>(
        sm, key, NeighbourDeltas<ITEMS>{key, heads, ahead}, bucket, present, 0ull, thr, (u32)P, 0ull, best_wait, bkey);
    if (!found) {
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
            rw.cr = nullptr; rw.narrow = false; rw.wide = false; rw.stride = 0; rw.k0 = rw.k1 = 0;
            int bad = 0;
            u64 best_wait = U64_MAX, best_rel = 0;
            // the 64-bit-delta form serves every deferred instance, narrow ones included
            // 64-bit keys: an instance of any value spread in one piece (or as few as its entries need)
            zl_window<NT, ITEMS, true, true>(sm, rw, thr, 0ull, range, best_wait, best_rel, bad);
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

}  // namespace

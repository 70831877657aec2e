// Front of the multi-window path: instance facts and fine-bin map, crossing indices, bin counts, windows.
// Part of the ZipLine library (see zipline.hip); device code for gfx950.
#pragma once
#include "zl_instance.h"

namespace {

// Multi-window path.

// zl_bounds: per-instance base, range, thr and the fine-bin grid.
template <int NT>
__global__ __launch_bounds__(NT) void zl_bounds_kernel(
    const i64* __restrict__ ts, const i64* __restrict__ le, const i64* __restrict__ iv, int P, int R, int bins,
    InstInfo* __restrict__ info, SegEntry* __restrict__ segtab, uint2* __restrict__ rowpar, int* __restrict__ status,
    bool summed, i64* __restrict__ best = nullptr)
{
    static_assert(NT >= SEGS, "one thread per segment");
    if (best && threadIdx.x == 0) best[blockIdx.x] = INT64_MAX;     // the instance's best upper bound so far (the sweep's slices share it)
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
    ii.wide_steps = 0;
    if (summed && ii.range > (u64)INT64_MAX / (u64)P) ii.flags |= EBSP_STATUS_OVERFLOW;    // P waits are summed
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
            slope = seg_slope_of(seg_est[tid], even, total2, bins, len);
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

// One wave walks one row: out[k] = number of entries of the row that fall in fine bins below k, for
// k = 0..nb (SUMS: every index written is also added to sums[k], an LDS array over the fine bins).  Every
// pair of neighbours is compared on the way (the only place the multi-window path does), and the steps
// of 2^32 or more of an instance whose values spread that far are remembered.  PART_AHEAD groups of 64
// entries are asked for before the first is looked at: a wave with one load in flight leaves the memory idle.
constexpr int PART_AHEAD = 4;
template <class CT, bool SUMS>
__device__ __forceinline__ void partition_row(const i64* __restrict__ row, int R, const InstInfo& ii, const SegEntry* tab,
                                              CT* __restrict__ out, u32* sums, i64 b, InstInfo* info, u32* __restrict__ widebin,
                                              int* __restrict__ status)
{
    const int lane = threadIdx.x & (WAVE - 1);
    const u64 base = (u64)ii.base;
    int carry = -1;                        // bin of the element before lane 0's
    i64 carry_t = INT64_MIN;               // and its value
    bool bad = false;
    const bool wide = (ii.range >> 32) != 0;          // only then can two neighbours be 2^32 or more apart
    int farbin = 0;                                   // the window kernels hold deltas in 32 bits: the bin such a
    u32 far = 0;                                      // step ends in is remembered (this lane's last one, and how many)
    for (u32 i0 = 0; i0 < (u32)R; i0 += PART_AHEAD * WAVE) {   // unsigned: R may be within a few waves' width of 2^31
        i64 tv[PART_AHEAD];
#pragma unroll
        for (int u = 0; u < PART_AHEAD; ++u) {
            const u32 i = i0 + (u32)(u * WAVE + lane);
            tv[u] = i < (u32)R ? row[i] : INT64_MAX;
        }
#pragma unroll
        for (int u = 0; u < PART_AHEAD; ++u) {
            const u32 i = i0 + (u32)(u * WAVE + lane);
            if (i0 + (u32)(u * WAVE) < (u32)R) {      // (the same in every lane)
                const i64 t = tv[u];
                int bin = -1;
                if (i < (u32)R) bin = (int)fine_bin((u64)t - base, ii, tab);
                // the neighbour's bin and value by a lane shift inside the vector ALU (lane 0: what the wave saw last)
                const int pb = dpp_take<DPP_WAVE_SHR1, 0xf>(carry, bin);
                const i64 pt = dpp_take<DPP_WAVE_SHR1, 0xf>(carry_t, t);
                bad |= t < pt;
                if (wide && i > 0 && i < (u32)R && (((u64)t - (u64)pt) >> 32) != 0) { farbin = bin; ++far; }
                if (i < (u32)R)
                    for (int k = pb + 1; k <= bin; ++k) {
                        out[k] = (CT)i;
                        if (SUMS) atomicAdd(&sums[k], i);
                    }
                carry = __builtin_amdgcn_readlane(bin, WAVE - 1);
                carry_t = (i64)((u64)(u32)__builtin_amdgcn_readlane((int)(u32)(u64)t, WAVE - 1) |
                                ((u64)(u32)__builtin_amdgcn_readlane((int)(u32)((u64)t >> 32), WAVE - 1) << 32));
            }
        }
    }
    if (__any(bad) && lane == 0 && status) atomicOr(status + b, (int)EBSP_STATUS_UNSORTED);
    if (far) {                                        // (a lane with several such steps: more than the list takes)
        const u32 slot = atomicAdd(&info[b].wide_steps, far == 1 ? 1u : WIDE_MARKS + 1u);
        if (far == 1 && slot < WIDE_MARKS) widebin[b * (i64)WIDE_MARKS + slot] = (u32)farbin;
    }
    const int last_bin = (int)fine_bin((u64)row[R - 1] - base, ii, tab);
    for (int k = last_bin + 1 + lane; k <= (int)ii.nb; k += WAVE) {
        out[k] = (CT)R;
        if (SUMS) atomicAdd(&sums[k], (u32)R);
    }
}

// zl_partition: one wave per row.  cross[row][k] = number of entries of the row
// that fall in fine bins below k, for k = 0..nb.
template <int NT, class CT>
__global__ __launch_bounds__(NT) void zl_partition_kernel(
    const i64* __restrict__ ts, i64 nrows, int P, int R,
    InstInfo* info, u32* __restrict__ widebin, const SegEntry* __restrict__ segtab, CT* __restrict__ cross, int stride,
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
    partition_row<CT, false>(ts + row_id * (i64)R, R, ii, tab, cross + row_id * (i64)stride, nullptr, b, info, widebin, status);
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
    InstInfo* info, u32* __restrict__ widebin, const SegEntry* __restrict__ segtab, CT* __restrict__ cross, int stride,
    u32* __restrict__ part, int* __restrict__ status)
{
    constexpr int NT = PART_ROWS * WAVE;
    __shared__ SegEntry tab[SEGS];
    __shared__ u32 sums[PART_MAX_STRIDE];
    const int tid = threadIdx.x;
    const i64 b = blockIdx.x / (u32)groups;
    const int g = (int)(blockIdx.x % (u32)groups);
    const int p = g * PART_ROWS + (tid >> 6);
    const InstInfo ii = info[b];
    if (tid < SEGS) tab[tid] = segtab[b * (i64)SEGS + tid];
    for (int k = tid; k <= (int)ii.nb; k += NT) sums[k] = 0;
    __syncthreads();
    if (p < P) {
        const i64 row_id = b * (i64)P + p;
        partition_row<CT, true>(ts + row_id * (i64)R, R, ii, tab, cross + row_id * (i64)stride, sums, b, info, widebin, status);
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
// KPT neighbouring bins per thread (1 or 2: one store for both indices; pays where an instance has bins for many workgroups)
template <class CT, int KPT>
__global__ __launch_bounds__(256) void zl_partition_pred_kernel(
    const i64* __restrict__ le, const i64* __restrict__ iv, int P, int R,
    const InstInfo* __restrict__ info, const SegEntry* __restrict__ segtab, CT* __restrict__ cross, int stride,
    u32* __restrict__ part)
{
    struct alignas(KPT * sizeof(CT)) Some { CT v[KPT]; };
    constexpr int PRED_BINS_PER_BLOCK = 256 * KPT;
    const u32 kblocks = (u32)(stride + PRED_BINS_PER_BLOCK - 1) / PRED_BINS_PER_BLOCK;
    const i64 b = blockIdx.x / kblocks;
    const int k = (int)(blockIdx.x % kblocks) * PRED_BINS_PER_BLOCK + KPT * (int)threadIdx.x;   // bins k .. k + KPT - 1 (stride is even)
    const int p_begin = (int)blockIdx.y * PRED_ROWS_PER_BLOCK;           // a slice of the rows per workgroup
    const int p_end = p_begin + PRED_ROWS_PER_BLOCK < P ? p_begin + PRED_ROWS_PER_BLOCK : P;
    const InstInfo ii = info[b];
    const i64* __restrict__ lep = le + b * (i64)P;
    const i64* __restrict__ ivp = iv + b * (i64)P;
    // Division by a row's interval, once per (row, bin), is most of this kernel's work: the rows' reciprocals
    // (row_reciprocal) are taken once per workgroup.
    __shared__ u32 inv[PRED_ROWS_PER_BLOCK];
    if ((int)threadIdx.x < p_end - p_begin) inv[threadIdx.x] = row_reciprocal((u64)ivp[p_begin + (int)threadIdx.x]);   // 0: divide the long way
    __syncthreads();
    if (k > (int)ii.nb) return;
    const bool broken = (ii.flags & EBSP_STATUS_UNSORTED) != 0;      // a negative interval: indices stay zero
    // bin nb and beyond (the row's padding): everything lies below
    u64 edge[KPT];
#pragma unroll
    for (int j = 0; j < KPT; ++j)
        edge[j] = k + j >= (int)ii.nb ? U64_MAX : fine_bin_start((u32)(k + j), ii, segtab + b * (i64)SEGS);
    CT* __restrict__ out = cross + (b * (i64)P) * stride + k;
    const bool narrow_values = (ii.range >> 32) == 0;
    u32 sum[KPT] = {};
    for (int p = p_begin; p < p_end; ++p) {
        const u64 step = (u64)ivp[p];
        const u64 first = (u64)lep[p] + step - (u64)ii.base;
        const u32 m = inv[p - p_begin];
        Some c;
#pragma unroll
        for (int j = 0; j < KPT; ++j) {
            u64 below;                                               // entries with first + i * step < edge
            if (broken) below = 0;
            else if (edge[j] == U64_MAX) below = (u64)R;
            else if (edge[j] <= first) below = 0;
            else if (step == 0) below = (u64)R;
            else if (narrow_values && (step >> 32) == 0) {
                const u32 n = (u32)(edge[j] - first) - 1u;
                const u32 q = m ? div_by_reciprocal(n, (u32)step, m) : n / (u32)step;     // (no reciprocal: an interval of 1)
                below = (u64)q + 1u;
            }
            else below = (edge[j] - first - 1) / step + 1;
            const u32 cj = (u32)(below < (u64)R ? below : (u64)R);
            c.v[j] = (CT)cj;
            sum[j] += cj;
        }
        *(Some*)(out + (i64)p * stride) = c;
    }
    u32* __restrict__ mine = part + (b * (i64)gridDim.y + blockIdx.y) * stride + k;      // this slice's share of the column sums
#pragma unroll
    for (int j = 0; j < KPT; ++j) mine[j] = sum[j];
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
// which the window kernel leaves to the general search).  The greedy chain of window
// starts is followed by pointer doubling over the bins held in LDS, a slice of them at a
// time (see the kernel); the per-window values follow in parallel.  Per window: its first
// fine bin (winstart), its first and last value and the constants of the linear bucket map
// over that span (winval).
struct WinVal {
    u64 A, Elast;
    u64 inv52;     // floor(2^52 / scale)
    u32 scale;     // linear_scale(Elast - A, buckets); 0: not for the fast search (the window is 2^32 or more
                   // wide, or a row steps by 2^32 or more into it)
    u32 pad_;
};

template <int NT, int PLAN_SLICE>       // PLAN_SLICE: fine bins held in LDS at a time
__global__ __launch_bounds__(NT) void zl_plan_kernel(
    InstInfo* __restrict__ info, const SegEntry* __restrict__ segtab, const u32* __restrict__ below, int stride,
    const u32* __restrict__ widebin, bool pred, u32* __restrict__ winstart, WinVal* __restrict__ winval, int max_win,
    u32 fill, u32 buckets)
{
    __shared__ u32 ends[PLAN_SLICE + 1];   // ends[i + 1] = keys under bin k0 + i + 1 = where bin k0 + i ends
    __shared__ u32 found_all, slice_cnt, slice_last;
    __shared__ SegEntry tab[SEGS];         // the instance's fine-bin map
    __shared__ u16 hop[2][PLAN_SLICE + 1];
    __shared__ u64 vstart[PLAN_SLICE + 1]; // wide instances: the first value of bin k0 + i (range + 1 for bin nb)
    const int tid = threadIdx.x;
    const i64 b = blockIdx.x;
    const u32* bel = below + b * (i64)stride;
    u32* ws = winstart + b * (i64)(max_win + 1);
    WinVal* wv = winval + b * (i64)max_win;
    const InstInfo ii = info[b];
    const int nb = (int)ii.nb;
    static_assert(PLAN_SLICE % NT == 0, "whole ranks per thread");
    constexpr int RANKS = PLAN_SLICE / NT;              // ranks per thread: every window holds at least one bin
    // The bins are taken a slice at a time.  Inside a slice, jump[k] = the bin that opens the next
    // window if one opens at bin k (cnt: none in this slice); the windows open at s0, jump[s0],
    // jump[jump[s0]], ...  Thread r finds the r-th of them by squaring the jump table: level l applies
    // jump^(2^l) to the ranks with bit l set.  The window that is open at the end of a slice goes on
    // into the next one, whose s0 is the first bin that no longer fits it.
    // In an instance whose value spread is 2^32 or more a window also ends where it would get wider
    // than that: the fast window search holds keys relative to the window's first value in 32 bits.
    const bool wide = (ii.range >> 32) != 0;
    constexpr u64 SPAN_MAX = 1ull << 32;   // first value of the bin behind a window - first value of the window
    if (tid < SEGS) tab[tid] = segtab[b * (i64)SEGS + tid];
    u32 found = 0, open_key = 0;           // windows so far; keys under the first bin of the window that is open
    u64 open_start = 0;                    // wide: that bin's first value
    bool have_open = false;
    u16* jump = hop[0];
    u16* other = hop[1];
    for (int k0 = 0; k0 < nb; k0 += PLAN_SLICE) {
        const int cnt = nb - k0 < PLAN_SLICE ? nb - k0 : PLAN_SLICE;
        __syncthreads();                                  // the slice before is done with
#pragma unroll 4
        for (int i = tid; i <= cnt; i += NT) ends[i] = bel[k0 + i];
        if (tid == 0) { slice_cnt = 0; slice_last = 0; }
        __syncthreads();                                  // (the first time round also: tab is there)
        if (wide) {
            for (int i = tid; i <= cnt; i += NT)
                vstart[i] = k0 + i < nb ? fine_bin_start((u32)(k0 + i), ii, tab) : ii.range + 1;
            __syncthreads();
        }
        int s0 = 0;
        if (have_open) {                                  // first bin whose end lies more than `fill` past the open window's start
            const u32 limit = open_key + fill;            // no overflow: fill and the key count are both below 2^31
            int lo = 0, hi = cnt;
            while (lo < hi) {
                const int m = (lo + hi) >> 1;
                if (ends[m + 1] > limit || (wide && vstart[m + 1] - open_start > SPAN_MAX)) hi = m; else lo = m + 1;
            }
            s0 = lo;
        }
        if (s0 >= cnt) continue;                          // the same for every thread: the open window takes the whole slice
        for (int k = tid; k <= cnt; k += NT) {
            int lo = k + 1, hi = cnt;                     // first bin j > k whose end lies more than `fill` past the start of bin k
            if (k < cnt) {
                const u32 limit = ends[k] + fill;
                const u64 from = wide ? vstart[k] : 0ull;
                while (lo < hi) {
                    const int m = (lo + hi) >> 1;
                    if (ends[m + 1] > limit || (wide && vstart[m + 1] - from > SPAN_MAX)) hi = m; else lo = m + 1;
                }
            } else lo = cnt;
            jump[k] = (u16)lo;
        }
        u32 pos[RANKS];
#pragma unroll
        for (int q = 0; q < RANKS; ++q) pos[q] = (u32)s0;
        const u32 top_rank = (u32)cnt < (u32)max_win ? (u32)cnt : (u32)max_win;
        int level = 0;
        for (; (1u << level) <= top_rank; ++level) {
            __syncthreads();
#pragma unroll
            for (int q = 0; q < RANKS; ++q)
                if (((u32)(q * NT + tid) >> level) & 1u) pos[q] = jump[pos[q]];
            for (int k = tid; k <= cnt; k += NT) other[k] = jump[jump[k]];
            u16* t = jump; jump = other; other = t;
        }
        const u32 rank_end = 1u << level;                 // ranks from here on had their upper bits ignored: not windows
#pragma unroll
        for (int q = 0; q < RANKS; ++q) {
            const u32 r = (u32)(q * NT + tid);
            if (pos[q] < (u32)cnt && r < rank_end) {
                // more starts than max_win cannot come from sorted rows; the last window then runs to the end
                if (found + r < (u32)max_win) ws[found + r] = (u32)k0 + pos[q];
                atomicMax(&slice_cnt, r + 1);
            }
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < RANKS; ++q)
            if (pos[q] < (u32)cnt && (u32)(q * NT + tid) + 1 == slice_cnt) slice_last = pos[q];   // the slice's last window stays open
        __syncthreads();
        open_key = ends[slice_last];
        if (wide) open_start = vstart[slice_last];
        have_open = true;
        found += slice_cnt;
    }
    if (tid == 0) {
        const u32 nwin = found < (u32)max_win ? found : (u32)max_win;
        ws[nwin] = (u32)nb;
        info[b].nwin = nwin;
        found_all = nwin;
    }
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
        bool slow = (span >> 32) != 0;
        if (wide) {
            // predicted rows of such an instance are not for the fast search (their first values and intervals
            // are kept as 32-bit words); nor is an instance with more steps of 2^32 or more than the list of
            // the bins they end in holds (zl_partition's); else the windows with such a bin
            const u32 steps = ii.wide_steps;
            slow |= pred || steps > WIDE_MARKS;
            const u32 marks = steps <= WIDE_MARKS ? steps : 0u;
            const u32 k_lo = ws[j], k_hi = j + 1 < nwin ? ws[j + 1] : (u32)nb;
            for (u32 m = 0; m < marks; ++m) {
                const u32 kb = widebin[b * (i64)WIDE_MARKS + m];
                if (kb >= k_lo && kb < k_hi) slow = true;
            }
        }
        if (slow) v.scale = 0;
        wv[j] = v;
    }
}

}  // namespace

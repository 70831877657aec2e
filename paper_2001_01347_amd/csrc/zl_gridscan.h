// GridScan and FullGridScan: the paper's heuristic and exhaustive-ish comparators of the search.
// Part of the ZipLine library (see zipline.hip); device code for gfx950.
#pragma once
#include "zl_sweep.h"

namespace {

// Section IV, Algorithm 1 ("GridScan") and the paragraph "FullGridScan".  For a designated point e
// (an entry of a designated row) the set Z holds e and every other row's point nearest to e;
// d_Z = max(Z) - min(Z).  GridScan designates the row with the smallest first timestamp and keeps
// the smallest d_Z over its R points; FullGridScan designates every row in turn (n*R sets).  The
// paper scans a whole row for the nearest point; rows are sorted, so here it is a bisection: the
// last point below e and the first at or above it are the only candidates (the earlier one when
// both are equally near).
//   zl_gridscan_kernel         one workgroup per (instance, designated row): a thread per designated
//                              point keeps max(Z) and min(Z) while the workgroup goes through the other
//                              rows, each staged in LDS once (rows of up to GRID_RMAX entries) and
//                              searched there by all threads; first minimum over the points.
//   zl_gridscan_finish_kernel  first minimum over the designated rows, then Z* itself: every row's
//                              nearest point to the winning e (of equal timestamps the first),
//                              barrier = max(Z*), iters[p] = 1 + index of the point.
// Of equal d_Z the set met first in (row, point) order is kept, as a loop with a strict "<" would.

constexpr int GRID_NT = 256;
constexpr int GRID_JPT = 16;                 // designated points a thread handles at a time
constexpr int GRID_RMAX = 4096;              // longest row that is staged in LDS

struct GridBest {      // best designated point of one designated row
    u64 d;             // max(Z) - min(Z)
    u32 row, point;
};

// Value of the point of a sorted row (R entries, in LDS or global memory) nearest to e.
__device__ __forceinline__ i64 grid_nearest(const i64* row, u32 R, i64 e)
{
    u32 lo = 0, hi = R;                      // first index with row[i] >= e
    while (lo < hi) {
        const u32 m = lo + ((hi - lo) >> 1);
        if (row[m] < e) lo = m + 1; else hi = m;
    }
    if (lo == 0) return row[0];
    const i64 below = row[lo - 1];
    if (lo == R) return below;
    const i64 above = row[lo];
    return (u64)e - (u64)below <= (u64)above - (u64)e ? below : above;
}

// Index of that point: of equal timestamps the first.
__device__ __forceinline__ u32 grid_nearest_index(const i64* __restrict__ row, u32 R, i64 e)
{
    auto first_at_or_above = [&](i64 v) {
        u32 lo = 0, hi = R;
        while (lo < hi) {
            const u32 m = lo + ((hi - lo) >> 1);
            if (row[m] < v) lo = m + 1; else hi = m;
        }
        return lo;
    };
    const u32 up = first_at_or_above(e);
    if (up == 0) return 0;
    const u32 down = first_at_or_above(row[up - 1]);
    if (up == R) return down;
    return (u64)e - (u64)row[down] <= (u64)row[up] - (u64)e ? down : up;
}

__global__ __launch_bounds__(GRID_NT) void zl_gridscan_kernel(
    const i64* __restrict__ ts, int P, int R, int full, GridBest* __restrict__ best, int* __restrict__ status)
{
    __shared__ i64 staged[GRID_RMAX];
    __shared__ u64 red[3 * (GRID_NT / WAVE)];
    constexpr int NW = GRID_NT / WAVE;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid >> 6;
    const int designated = full ? P : 1;
    const i64 b = blockIdx.x / (u32)designated;
    const i64* __restrict__ inst = ts + b * (i64)P * R;
    int pb = (int)(blockIdx.x % (u32)designated);
    if (!full) {
        // the row with the smallest first timestamp (of several the first)
        i64 f = INT64_MAX;
        u32 who = 0xffffffffu;
        for (int p = tid; p < P; p += GRID_NT) {
            const i64 v = inst[(size_t)p * R];
            if (v < f) { f = v; who = (u32)p; }                // (p grows: the first of equal values stays)
        }
        u64 w = (u64)f ^ (1ull << 63);                          // order-preserving map to unsigned
        wave_argmin(w, who);
        if (lane == WAVE - 1) { red[wave] = w; red[NW + wave] = who; }
        __syncthreads();
        w = red[0]; who = (u32)red[NW];
        for (int k = 1; k < NW; ++k) {
            const u64 ow = red[k];
            const u32 ok = (u32)red[NW + k];
            if (ow < w || (ow == w && ok < who)) { w = ow; who = ok; }
        }
        pb = (int)who;
        __syncthreads();
    }
    const bool lds_rows = R <= GRID_RMAX;
    const bool checker = status != nullptr && blockIdx.x % (u32)designated == 0;   // one workgroup per instance checks the rows' order
    int bad = 0;
    u64 bd = U64_MAX;
    u32 bj = 0xffffffffu;
    const i64* __restrict__ drow = inst + (size_t)pb * R;
    for (u32 j0 = 0; j0 < (u32)R; j0 += GRID_NT * GRID_JPT) {
        i64 e[GRID_JPT], mx[GRID_JPT], mn[GRID_JPT];
#pragma unroll
        for (int k = 0; k < GRID_JPT; ++k) {
            const u32 j = j0 + (u32)k * GRID_NT + tid;
            e[k] = j < (u32)R ? drow[j] : 0;
            mx[k] = mn[k] = e[k];
        }
        for (int p = 0; p < P; ++p) {
            const i64* __restrict__ row = inst + (size_t)p * R;
            if (lds_rows) {
                __syncthreads();                                  // the row staged before has been searched
                for (int i = tid; i < R; i += GRID_NT) staged[i] = row[i];
                __syncthreads();
                if (checker && j0 == 0)
                    for (int i = tid + 1; i < R; i += GRID_NT) bad |= staged[i] < staged[i - 1];
            } else if (checker && j0 == 0) {
                for (int i = tid + 1; i < R; i += GRID_NT) bad |= row[i] < row[i - 1];
            }
            if (p == pb) continue;
            const i64* look = lds_rows ? staged : row;
#pragma unroll
            for (int k = 0; k < GRID_JPT; ++k) {
                const u32 j = j0 + (u32)k * GRID_NT + tid;
                if (j < (u32)R) {
                    const i64 v = grid_nearest(look, (u32)R, e[k]);
                    mx[k] = v > mx[k] ? v : mx[k];
                    mn[k] = v < mn[k] ? v : mn[k];
                }
            }
        }
#pragma unroll
        for (int k = 0; k < GRID_JPT; ++k) {
            const u32 j = j0 + (u32)k * GRID_NT + tid;
            if (j < (u32)R) {
                const u64 d = (u64)mx[k] - (u64)mn[k];
                if (d < bd || (d == bd && j < bj)) { bd = d; bj = j; }
            }
        }
    }
    // first minimum over the designated points: smaller d_Z, then the earlier point
    wave_argmin(bd, bj);
    __syncthreads();
    if (lane == WAVE - 1) { red[wave] = bd; red[NW + wave] = bj; }
    bad = __syncthreads_or(bad);
    if (tid == 0) {
        u64 w = red[0];
        u32 j = (u32)red[NW];
        for (int k = 1; k < NW; ++k) {
            const u64 ow = red[k];
            const u32 oj = (u32)red[NW + k];
            if (ow < w || (ow == w && oj < j)) { w = ow; j = oj; }
        }
        GridBest r;
        r.d = w;
        r.row = (u32)pb;
        r.point = j;
        best[blockIdx.x] = r;
        if (checker) status[b] = bad ? (int)EBSP_STATUS_UNSORTED : 0;
    }
}

__global__ __launch_bounds__(GRID_NT) void zl_gridscan_finish_kernel(
    const i64* __restrict__ ts, int P, int R, int full, const GridBest* __restrict__ best,
    i64* __restrict__ barrier, int* __restrict__ iters, i64* __restrict__ dz)
{
    __shared__ u64 red[3 * (GRID_NT / WAVE)];
    constexpr int NW = GRID_NT / WAVE;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid >> 6;
    const i64 b = blockIdx.x;
    const int designated = full ? P : 1;
    const GridBest* mine = best + b * (i64)designated;
    // first minimum over the designated rows: smaller d_Z, then the earlier row (its point is its own first minimum)
    u64 bd = U64_MAX;
    u32 bq = 0xffffffffu;
    for (int q = tid; q < designated; q += GRID_NT) {
        const u64 d = mine[q].d;
        if (d < bd) { bd = d; bq = (u32)q; }
    }
    wave_argmin(bd, bq);
    if (lane == WAVE - 1) { red[wave] = bd; red[NW + wave] = bq; }
    __syncthreads();
    bd = red[0]; bq = (u32)red[NW];
    for (int k = 1; k < NW; ++k) {
        const u64 od = red[k];
        const u32 oq = (u32)red[NW + k];
        if (od < bd || (od == bd && oq < bq)) { bd = od; bq = oq; }
    }
    __syncthreads();
    const GridBest win = mine[bq];
    const i64* __restrict__ inst = ts + b * (i64)P * R;
    const i64 e = inst[(size_t)win.row * R + win.point];
    i64 mx = e;
    for (int p = tid; p < P; p += GRID_NT) {
        const i64* __restrict__ row = inst + (size_t)p * R;
        const u32 i = (u32)p == win.row ? win.point : grid_nearest_index(row, (u32)R, e);
        iters[b * (i64)P + p] = (int)i + 1;
        const i64 v = row[i];
        mx = v > mx ? v : mx;
    }
    const i64 top = block_reduce<i64, GRID_NT>(mx, (i64*)red, OpMax());
    if (tid == 0) { barrier[b] = top; dz[b] = (i64)win.d; }
}

}  // namespace

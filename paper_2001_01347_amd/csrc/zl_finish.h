// Reduction of the window results, iteration counts; the copy kernel used as a yardstick.
// Part of the ZipLine library (see zipline.hip); device code for gfx950.
#pragma once
#include "zl_range.h"

namespace {

// zl_iters for the multi-window path: reduce the instance's window results
// (first minimum: smaller wait, then earlier barrier), then count iterations.  For stored
// rows the crossing indices of the barrier's fine bin bracket the count, so the binary
// search runs over the row's few entries of that bin instead of the whole row.
template <int NT>
__global__ __launch_bounds__(NT) void zl_finish_kernel(
    const i64* __restrict__ ts, const i64* __restrict__ le, const i64* __restrict__ iv, int P, int R,
    const InstInfo* __restrict__ info, const SegEntry* __restrict__ segtab, const void* __restrict__ cross, bool narrow,
    int stride, const Partial* __restrict__ partial, int max_win,
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
    if (p >= P) return;
    if (!ts) {
        iters[b * (i64)P + p] = zl_iters_of(nullptr, le + b * (i64)P, iv + b * (i64)P, p, R, bar);
        return;
    }
    Rows rw;                                     // only for the index range of row p inside the barrier's fine bin
    rw.R = R;
    rw.cr = narrow ? (const void*)((const unsigned short*)cross + (b * (i64)P) * stride)
                   : (const void*)((const u32*)cross + (b * (i64)P) * stride);
    rw.narrow = narrow;
    rw.stride = stride;
    rw.k0 = fine_bin(bb, ii, segtab + b * (i64)SEGS);
    rw.k1 = rw.k0 + 1;                           // k0 < nb, and a row of cross holds nb + 1 indices
    u32 lo, hi;
    rw.range(p, lo, hi);                         // entries before lo lie in lower bins (<= barrier), from hi on in higher ones
    const i64* __restrict__ row = ts + (b * (i64)P + p) * (i64)R;
    while (lo < hi) {
        const u32 m = (lo + hi) >> 1;
        if (row[m] <= bar) lo = m + 1; else hi = m;
    }
    iters[b * (i64)P + p] = (int)lo;
}

// Superstep simulation: after a barrier (and the synchronisation, which takes sync_cost) every
// worker of an instance starts its next iteration together.  start[b][p] = barrier[b] + sync_cost;
// an instance whose search raised a status bit has no barrier: its workers keep `from`, the times
// they started the superstep at.
__global__ __launch_bounds__(256) void zl_advance_kernel(const i64* __restrict__ barrier, const int* __restrict__ status,
                                                         const i64* from, i64* start,
                                                         i64 sync_cost, i64 B, int P)
{
    const i64 at = (i64)blockIdx.x * 256 + threadIdx.x;
    if (at >= B * (i64)P) return;
    const i64 b = at / P;
    start[at] = (!status || status[b] == 0) ? barrier[b] + sync_cost : from[at];
}

// Plain streaming copy of n 16-byte words: the yardstick that HBM byte counters and achieved bandwidth of the
// other kernels are read against.  Every workgroup takes one contiguous piece, four 16-byte loads in flight per
// lane (pieces that follow each other in memory go to workgroups that follow each other: the order in which the
// memory likes to be read; a grid-wide stride between a lane's loads reaches three quarters of this speed).
constexpr int PROBE_AHEAD = 4;
__global__ __launch_bounds__(256) void zl_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, i64 n)
{
    const i64 per = (n + gridDim.x - 1) / gridDim.x;
    const i64 b0 = (i64)blockIdx.x * per, b1 = b0 + per < n ? b0 + per : n;
    i64 i = b0 + threadIdx.x;
    for (; i + (PROBE_AHEAD - 1) * 256 < b1; i += PROBE_AHEAD * 256) {
        uint4 v[PROBE_AHEAD];
#pragma unroll
        for (int k = 0; k < PROBE_AHEAD; ++k) v[k] = src[i + k * 256];
#pragma unroll
        for (int k = 0; k < PROBE_AHEAD; ++k) dst[i + k * 256] = v[k];
    }
    for (; i < b1; i += 256) dst[i] = src[i];
}

// Plain streaming read of n 16-byte words in the same order; every workgroup adds the sum of its words to
// sink[blockIdx.x % READ_SINK_WORDS] so that no load can be dropped.  The yardstick for kernels that read far
// more than they write.
constexpr int READ_SINK_WORDS = 256;
__global__ __launch_bounds__(256) void zl_read_kernel(const uint4* __restrict__ src, i64 n, u64* __restrict__ sink)
{
    __shared__ u64 red[4];
    const i64 per = (n + gridDim.x - 1) / gridDim.x;
    const i64 b0 = (i64)blockIdx.x * per, b1 = b0 + per < n ? b0 + per : n;
    i64 i = b0 + threadIdx.x;
    u64 acc = 0;
    for (; i + (PROBE_AHEAD - 1) * 256 < b1; i += PROBE_AHEAD * 256) {
        uint4 v[PROBE_AHEAD];
#pragma unroll
        for (int k = 0; k < PROBE_AHEAD; ++k) v[k] = src[i + k * 256];
#pragma unroll
        for (int k = 0; k < PROBE_AHEAD; ++k) acc += (u64)v[k].x + v[k].y + v[k].z + v[k].w;
    }
    for (; i < b1; i += 256) {
        const uint4 a = src[i];
        acc += (u64)a.x + a.y + a.z + a.w;
    }
    acc = block_reduce<u64, 256>(acc, red, OpAdd());
    if (threadIdx.x == 0) atomicAdd(sink + blockIdx.x % READ_SINK_WORDS, acc);
}

}  // namespace

// Types, constants, per-instance records, wave and block primitives (wave64), the fine-bin map.
// Part of the ZipLine library (see zipline.hip); device code for gfx950.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <limits>

#include "ebsp_zipline.h"

#define ZL_FN __host__ __device__ __forceinline__
#include "zl_maps.h"


namespace {

constexpr int WAVE = 64;
constexpr u64 U64_MAX = ~0ull;
constexpr i64 DEFERRED = INT64_MIN;            // wait[b] of an instance left to the general kernel
constexpr u64 DEFERRED_WINDOW = ~0ull - 1;      // Partial::brel of a window left to the general kernel

// ---------------------------------------------------------------------------
// Tunables of the multi-window path.
constexpr int LARGE_NT = 1024;               // threads of a general-path workgroup
constexpr int LARGE_ITEMS = 16;              // records per thread
constexpr int SINGLE_MAX = LARGE_NT * LARGE_ITEMS;  // largest P*R one workgroup takes whole
constexpr int GENERAL_GRID = 256;            // workgroups of a general-path kernel (one per CU)
// A window workgroup holds up to `cap` records (4096, 8192 or 16384).  Windows are
// packed, as full as that allows, out of fine bins that hold about cap/8 keys each.

struct Partial {  // best candidate of one window
    u64 wait;     // U64_MAX: the window has no admissible candidate
    u64 brel;     // barrier relative to base
};

// ---------------------------------------------------------------------------
// Wave and block primitives (wave64).

// Cross-lane moves inside the vector ALU (data-parallel primitives): no trip
// through the LDS pipeline.  dpp_take<CTRL, ROWS>(fill, v) gives every lane the
// value of the lane that CTRL selects; lanes in rows outside the ROWS mask and
// lanes whose source does not exist get `fill`.
template <int CTRL, int ROWS>
__device__ __forceinline__ u32 dpp_word(u32 fill, u32 v)
{
    return (u32)__builtin_amdgcn_update_dpp((int)fill, (int)v, CTRL, ROWS, 0xf, false);
}
template <int CTRL, int ROWS, class T>
__device__ __forceinline__ T dpp_take(T fill, T v)
{
    static_assert(sizeof(T) == 4 || sizeof(T) == 8, "one or two words");
    if constexpr (sizeof(T) == 4) {
        return (T)dpp_word<CTRL, ROWS>((u32)fill, (u32)v);
    } else {
        const u64 f = (u64)fill, x = (u64)v;
        return (T)((u64)dpp_word<CTRL, ROWS>((u32)f, (u32)x) |
                   ((u64)dpp_word<CTRL, ROWS>((u32)(f >> 32), (u32)(x >> 32)) << 32));
    }
}
constexpr int DPP_ROW_SHR1 = 0x111, DPP_ROW_SHR2 = 0x112, DPP_ROW_SHR4 = 0x114, DPP_ROW_SHR8 = 0x118,
              DPP_ROW_BCAST15 = 0x142, DPP_ROW_BCAST31 = 0x143,
              DPP_WAVE_SHR1 = 0x138;      // every lane takes the value of the lane before it (across rows)

// A value that all lanes of a wave hold alike, moved to scalar registers.
__device__ __forceinline__ u32 uniform(u32 x) { return (u32)__builtin_amdgcn_readfirstlane((int)x); }
__device__ __forceinline__ u64 uniform(u64 x) { return (u64)uniform((u32)x) | ((u64)uniform((u32)(x >> 32)) << 32); }

// The value that lane 63 holds, for every lane (scalar registers).
__device__ __forceinline__ u32 last_lane(u32 x) { return (u32)__builtin_amdgcn_readlane((int)x, WAVE - 1); }
__device__ __forceinline__ u64 last_lane(u64 x) { return (u64)last_lane((u32)x) | ((u64)last_lane((u32)(x >> 32)) << 32); }

struct OpMin {
    template <class T> __device__ T operator()(T a, T b) const { return a < b ? a : b; }
    template <class T> static constexpr T identity() { return std::numeric_limits<T>::max(); }
};
struct OpMax {
    template <class T> __device__ T operator()(T a, T b) const { return a > b ? a : b; }
    template <class T> static constexpr T identity() { return std::numeric_limits<T>::lowest(); }
};
struct OpAdd {
    template <class T> __device__ T operator()(T a, T b) const { return a + b; }
    template <class T> static constexpr T identity() { return T(0); }
};

// Inclusive scan over the 64 lanes of a wave: four steps inside each row of 16
// lanes, then the row totals are passed on (last lane of row 0 and 2 to rows 1
// and 3, last lane of row 1 to rows 2 and 3).  Lane 63 ends with the reduction.
template <class T, class Op>
__device__ __forceinline__ T wave_scan(T v, Op op)
{
    constexpr T id = Op::template identity<T>();
    v = op(v, dpp_take<DPP_ROW_SHR1, 0xf>(id, v));
    v = op(v, dpp_take<DPP_ROW_SHR2, 0xf>(id, v));
    v = op(v, dpp_take<DPP_ROW_SHR4, 0xf>(id, v));
    v = op(v, dpp_take<DPP_ROW_SHR8, 0xf>(id, v));
    v = op(v, dpp_take<DPP_ROW_BCAST15, 0xa>(id, v));
    v = op(v, dpp_take<DPP_ROW_BCAST31, 0xc>(id, v));
    return v;
}
template <class T>
__device__ __forceinline__ T wave_incl_scan(T v) { return wave_scan(v, OpAdd()); }

// First minimum of (w, k) pairs over a wave (smaller w, then smaller k); lane 63 ends with it.
template <class K>
__device__ __forceinline__ void wave_argmin(u64& w, K& k)
{
    auto step = [&](u64 ow, K ok) { if (ow < w || (ow == w && ok < k)) { w = ow; k = ok; } };
    constexpr K kmax = std::numeric_limits<K>::max();
    step(dpp_take<DPP_ROW_SHR1, 0xf>(U64_MAX, w), dpp_take<DPP_ROW_SHR1, 0xf>(kmax, k));
    step(dpp_take<DPP_ROW_SHR2, 0xf>(U64_MAX, w), dpp_take<DPP_ROW_SHR2, 0xf>(kmax, k));
    step(dpp_take<DPP_ROW_SHR4, 0xf>(U64_MAX, w), dpp_take<DPP_ROW_SHR4, 0xf>(kmax, k));
    step(dpp_take<DPP_ROW_SHR8, 0xf>(U64_MAX, w), dpp_take<DPP_ROW_SHR8, 0xf>(kmax, k));
    step(dpp_take<DPP_ROW_BCAST15, 0xa>(U64_MAX, w), dpp_take<DPP_ROW_BCAST15, 0xa>(kmax, k));
    step(dpp_take<DPP_ROW_BCAST31, 0xc>(U64_MAX, w), dpp_take<DPP_ROW_BCAST31, 0xc>(kmax, k));
}

// Exclusive block scan; `total` receives the block sum.  `red` holds NT/64 T's.
template <class T, int NT>
__device__ __forceinline__ T block_excl_scan(T v, T* red, T& total)
{
    constexpr int NW = NT / WAVE;
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x >> 6;
    T inc = wave_incl_scan(v);
    if (lane == WAVE - 1) red[wave] = inc;
    __syncthreads();
    T base = 0, sum = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        T x = red[w];
        if (w < wave) base += x;
        sum += x;
    }
    __syncthreads();
    total = sum;
    return base + inc - v;
}

template <class T, int NT, class Op>
__device__ __forceinline__ T block_reduce(T v, T* red, Op op)
{
    constexpr int NW = NT / WAVE;
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x >> 6;
    v = wave_scan(v, op);
    if (lane == WAVE - 1) red[wave] = v;
    __syncthreads();
    T r = red[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) r = op(r, red[w]);
    asm volatile("" : "+v"(r));      // finish the reduction here, not wherever the result is first used
    __syncthreads();
    return r;
}

// min of a, max of b, max of c over the block in one exchange.  `red` holds 3*NT/64 words.
template <int NT>
__device__ __forceinline__ void block_bounds(i64 a, i64 b, i64 c, i64* red, i64& amin, i64& bmax, i64& cmax)
{
    constexpr int NW = NT / WAVE;
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x >> 6;
    a = wave_scan(a, OpMin());
    b = wave_scan(b, OpMax());
    c = wave_scan(c, OpMax());
    if (lane == WAVE - 1) { red[wave] = a; red[NW + wave] = b; red[2 * NW + wave] = c; }
    __syncthreads();
    a = red[0]; b = red[NW]; c = red[2 * NW];
#pragma unroll
    for (int w = 1; w < NW; ++w) {
        const i64 oa = red[w], ob = red[NW + w], oc = red[2 * NW + w];
        a = oa < a ? oa : a;
        b = ob > b ? ob : b;
        c = oc > c ? oc : c;
    }
    __syncthreads();
    amin = a; bmax = b; cmax = c;
}

}  // namespace

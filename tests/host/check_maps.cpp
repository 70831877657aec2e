// Host check of the integer maps the GPU search prunes with (paper_2001_01347_amd/csrc/zl_maps.h): compiled with g++
// and run by tests/test_host_maps.py.  Every property is checked against exact arithmetic (128-bit products and
// divisions, or a walk over every key), never against the functions' own formulas:
//   LinearMap / TableMap   lo(b) <= k <= hi(b) for every key k in [0, span] that the map sends to bucket b;
//                          the map never decreases and stays below the bucket count;
//   fine_bin               never decreases, ends at nb - 1;  fine_bin_start(k) is the smallest value of bin >= k.
// A bound that is too tight would drop a bucket holding the optimum: the search would still return a barrier, only
// not the best one, and parity tests would see it only on the inputs that happen to hit it.
#include <cstdio>
#include <cstdlib>
#include <vector>

#define ZL_FN inline
#include "../../paper_2001_01347_amd/csrc/zl_maps.h"

typedef unsigned __int128 u128;

static long long checks = 0, failures = 0;
#define FAIL(...)                                                 \
    do {                                                          \
        if (failures < 20) { std::printf("FAIL: " __VA_ARGS__); std::printf("\n"); } \
        ++failures;                                               \
    } while (0)

static u64 rng_state = 0x9e3779b97f4a7c15ull;
static u64 rnd()
{   // splitmix64
    u64 z = (rng_state += 0x9e3779b97f4a7c15ull);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return z ^ (z >> 31);
}

// ---------------------------------------------------------------- LinearMap
static void linear_case(u32 span, u32 nb, u32 scale, bool walk)
{
    const LinearMap m = linear_map(span, nb, scale, (1ull << 52) / scale);
    const u32 top = nb - 1;
    for (u32 b = 0; b <= top; ++b) {
        // exact keys of bucket b: k * scale in [b * 2^32, (b + 1) * 2^32), the last bucket takes the rest
        const u128 kmin128 = (((u128)b << 32) + scale - 1) / scale;
        if (kmin128 > span) break;                                   // bucket b and all later ones hold no key <= span
        const u64 kmin = (u64)kmin128;
        u64 kmax = b < top ? (u64)(((((u128)(b + 1)) << 32) + scale - 1) / scale) - 1 : span;
        if (kmax > span) kmax = span;
        if (m((u32)kmin) != b || m((u32)kmax) != b) FAIL("linear map: span %u nb %u scale %u bucket %u ends [%llu, %llu]", span, nb, scale, b, kmin, kmax);
        u32 lo, hi;
        m.bounds(b, lo, hi);
        ++checks;
        if (!(lo <= kmin && kmax <= hi && hi <= span)) FAIL("linear bounds: span %u nb %u scale %u bucket %u keys [%llu, %llu] bounds [%u, %u]", span, nb, scale, b, kmin, kmax, lo, hi);
        if (!(b & 1) && b + 1 <= top) {
            u32 lo0, hi0, lo1, hi1;
            m.bounds_pair(b, lo0, hi0, lo1, hi1);
            if (!(lo0 <= kmin && kmax <= hi0 && hi0 <= span)) FAIL("linear bounds_pair(first): span %u nb %u scale %u bucket %u keys [%llu, %llu] bounds [%u, %u]", span, nb, scale, b, kmin, kmax, lo0, hi0);
            const u128 k1min = (((u128)(b + 1) << 32) + scale - 1) / scale;
            if (k1min <= span) {
                u64 k1max = b + 1 < top ? (u64)(((((u128)(b + 2)) << 32) + scale - 1) / scale) - 1 : span;
                if (k1max > span) k1max = span;
                if (!(lo1 <= (u64)k1min && k1max <= hi1 && hi1 <= span)) FAIL("linear bounds_pair(second): span %u nb %u scale %u bucket %u keys [%llu, %llu] bounds [%u, %u]", span, nb, scale, b + 1, (u64)k1min, k1max, lo1, hi1);
            }
        }
    }
    if (walk) {                                                      // every key, one by one
        u32 prev = 0;
        for (u64 k = 0; k <= span; ++k) {
            const u32 b = m((u32)k);
            u32 lo, hi;
            m.bounds(b, lo, hi);
            ++checks;
            if (b > top || b < prev || k < lo || k > hi) FAIL("linear walk: span %u nb %u scale %u key %llu bucket %u bounds [%u, %u]", span, nb, scale, k, b, lo, hi);
            prev = b;
        }
    }
}

static void check_linear()
{
    const u32 nbs[] = {2, 3, 64, 512, 1024, 2048};
    std::vector<u32> spans;
    for (u32 s = 0; s <= 3000; ++s) spans.push_back(s);
    for (int e = 12; e <= 32; ++e)
        for (int d = -2; d <= 2; ++d) {
            const u64 v = (1ull << e) + d;
            if (v <= 0xffffffffull) spans.push_back((u32)v);
        }
    for (int i = 0; i < 20000; ++i) spans.push_back((u32)(rnd() >> (32 + rnd() % 21)));
    for (u32 nb : nbs)
        for (size_t i = 0; i < spans.size(); ++i) {
            const u32 span = spans[i];
            linear_case(span, nb, linear_scale(span, nb), span <= 3000);
            // a window left to the slower search keeps a map with scale 1; extreme scales for good measure
            if (i % 16 == 0) {
                linear_case(span, nb, 1u, span <= 3000);
                linear_case(span, nb, 0xffffffffu, span <= 3000);
                linear_case(span, nb, 0x80000000u, false);
                linear_case(span, nb, (u32)rnd() | 1u, false);
            }
        }
}

// ---------------------------------------------------------------- TableMap
static void table_case(const std::vector<u32>& keys, u32 range, u32 NB, bool walk)
{
    std::vector<u64> tab(512);
    TableMap<true> m;
    const int bl = bit_length(range);
    m.tab = tab.data();
    m.cshift = bl > 8 ? (u32)(bl - 8) : 0u;
    m.cmask = (1u << m.cshift) - 1u;
    m.span = range;
    u32 cnt[256] = {0};
    for (u32 k : keys) ++cnt[m.coarse(k)];
    u32 below = 0;
    for (int c = 0; c < 256; ++c) {
        table_entry(below, cnt[c], (u32)keys.size(), NB, m.cshift, tab[c], tab[256 + c]);
        below += cnt[c];
    }
    auto one = [&](u64 k, const char* what) {
        const u32 b = m((u32)k);
        u32 lo, hi;
        ++checks;
        if (b >= NB) { FAIL("table map (%s): range %u NB %u key %llu bucket %u", what, range, NB, k, b); return b; }
        m.bounds(b, lo, hi);
        if (k < lo || k > hi || hi > range) FAIL("table bounds (%s): range %u NB %u n %zu key %llu bucket %u bounds [%u, %u]", what, range, NB, keys.size(), k, b, lo, hi);
        if (!(b & 1) && b + 1 < NB) {
            u32 lo0, hi0, lo1, hi1;
            m.bounds_pair(b, lo0, hi0, lo1, hi1);
            if (lo0 != lo || hi0 != hi) FAIL("table bounds_pair: range %u NB %u bucket %u", range, NB, b);
        }
        return b;
    };
    for (u32 k : keys) one(k, "present key");
    if (walk) {
        u32 prev = 0;
        for (u64 k = 0; k <= range; ++k) {
            const u32 b = one(k, "walk");
            if (b < prev) FAIL("table map decreases: range %u NB %u key %llu", range, NB, k);
            prev = b;
        }
    } else {
        // around every coarse-bin edge and at random places
        for (u32 c = 0; c < 256; ++c)
            for (int d = -3; d <= 3; ++d) {
                const long long k = ((long long)c << m.cshift) + d;
                if (k >= 0 && k <= (long long)range) one((u64)k, "bin edge");
            }
        u32 prev_b = 0;
        u64 prev_k = 0;
        std::vector<u64> probes;
        for (int i = 0; i < 4000; ++i) probes.push_back(rnd() % ((u64)range + 1));
        // monotone over a sorted sample
        for (size_t i = 0; i < probes.size(); ++i)
            for (size_t j = i + 1; j < probes.size() && j < i + 2; ++j)
                if (probes[j] < probes[i]) { const u64 t = probes[i]; probes[i] = probes[j]; probes[j] = t; }
        for (u64 k : probes) {
            const u32 b = one(k, "probe");
            if ((k >= prev_k && b < prev_b) || (k <= prev_k && b > prev_b)) FAIL("table map not monotone: range %u NB %u keys %llu %llu", range, NB, prev_k, k);
            prev_k = k; prev_b = b;
        }
    }
}

static void check_table()
{
    const u32 ranges[] = {0, 1, 2, 100, 255, 256, 257, 511, 512, 1000, 4095, 65535, 65536, 70001, 1u << 20, (1u << 20) + 12345,
                          1u << 31, (1u << 31) - 1, 0xfffffffeu, 0xffffffffu};
    const u32 NBs[] = {128, 512, 1024, 2048};
    const u32 ns[] = {1, 2, 7, 300, 4096, 16384};
    for (u32 range : ranges)
        for (u32 NB : NBs)
            for (u32 n : ns)
                for (int dist = 0; dist < 7; ++dist) {
                    std::vector<u32> keys(n);
                    const u64 span1 = (u64)range + 1;
                    for (u32 i = 0; i < n; ++i) {
                        u64 k = 0;
                        switch (dist) {
                        case 0: k = rnd() % span1; break;                                  // uniform
                        case 1: k = 0; break;                                              // all at the low end
                        case 2: k = range; break;                                          // all at the high end
                        case 3: k = (range / 3 + rnd() % (span1 / 200 + 1)) % span1; break;   // one cluster
                        case 4: k = (i & 1) ? rnd() % (span1 / 50 + 1) : range - rnd() % (span1 / 50 + 1); break;   // both ends
                        case 5: k = range >> (rnd() % 33 > 31 ? 31 : rnd() % 32); break;   // geometric
                        default: k = (u64)((double)(i + 1) / n * range); break;             // evenly spaced, the last at range
                        }
                        keys[i] = (u32)k;
                    }
                    table_case(keys, range, NB, range <= 70001 && n != 4096);
                }
}

// ---------------------------------------------------------------- fine-bin grid
static void fine_case(u64 range, int bins, int kind)
{
    InstInfo ii{};
    ii.range = range;
    const int bl = bit_length(range);
    ii.wshift = bl > 32 ? (u32)(bl - 32) : 0u;
    const u64 top = range >> ii.wshift;
    const int tl = bit_length(top);
    ii.segshift = tl > 6 ? (u32)(tl - 6) : 0u;
    const u64 W = 1ull << ii.segshift;
    const int nseg = (int)(top >> ii.segshift) + 1;
    if (nseg > SEGS) { FAIL("fine grid: %d segments", nseg); return; }
    u64 est[SEGS] = {0}, total = 0;
    for (int s = 0; s < nseg; ++s) {
        switch (kind) {
        case 0: est[s] = 1000; break;
        case 1: est[s] = rnd() % 100000; break;
        case 2: est[s] = s == 0 ? 1ull << 40 : 0; break;                       // everything in the first segment
        case 3: est[s] = s == nseg - 1 ? 1ull << 40 : 0; break;                // everything in the last
        default: est[s] = (rnd() & 3) ? 0 : rnd() % (1ull << 36); break;       // sparse
        }
        total += est[s];
    }
    const u64 even = total / (8ull * (u64)nseg) + 1, total2 = total + even * (u64)nseg;
    SegEntry tab[SEGS] = {};
    u64 G = 0;
    for (int s = 0; s < SEGS; ++s) {
        u32 slope = 0;
        if (s < nseg) {
            const u64 len = s == nseg - 1 ? top - ((u64)s << ii.segshift) + 1 : W;
            slope = seg_slope_of(est[s], even, total2, bins, len);
        }
        tab[s].G = G;
        tab[s].slope = slope;
        if (s == nseg - 1) ii.nb = (u32)((G + (top - ((u64)s << ii.segshift)) * (u64)slope) >> 32) + 1u;
        G += W * (u64)slope;
    }
    ++checks;
    if (ii.nb < 1 || ii.nb > (u32)bins) FAIL("fine grid: range %llu bins %d kind %d gives nb %u", range, bins, kind, ii.nb);
    if (fine_bin(range, ii, tab) != ii.nb - 1 || fine_bin(0, ii, tab) != 0) FAIL("fine grid ends: range %llu bins %d kind %d", range, bins, kind);
    if (fine_bin(~0ull, ii, tab) != ii.nb - 1) FAIL("fine grid beyond the range: range %llu bins %d kind %d", range, bins, kind);
    // exact bin of x by 128-bit arithmetic, and the start of every bin
    const u64 unit = 1ull << ii.wshift;
    u64 prev_start = 0;
    for (u32 k = 0; k < ii.nb; ++k) {
        const u64 s = fine_bin_start(k, ii, tab);
        ++checks;
        if (s > range || (s & (unit - 1))) { FAIL("fine_bin_start: range %llu bins %d kind %d bin %u start %llu", range, bins, kind, k, s); continue; }
        if (fine_bin(s, ii, tab) < k) FAIL("fine_bin_start too early: range %llu bins %d kind %d bin %u start %llu (bin %u)", range, bins, kind, k, s, fine_bin(s, ii, tab));
        if (s >= unit && fine_bin(s - unit, ii, tab) >= k) FAIL("fine_bin_start too late: range %llu bins %d kind %d bin %u start %llu", range, bins, kind, k, s);
        if (s && fine_bin(s - 1, ii, tab) >= k) FAIL("fine_bin_start not the first of its unit: range %llu bin %u", range, k);
        if (s < prev_start) FAIL("fine_bin_start decreases: range %llu bin %u", range, k);
        if (k && ii.nb > 1 && s == prev_start && fine_bin(s, ii, tab) < k) FAIL("empty bin: range %llu bin %u", range, k);
        prev_start = s;
    }
    // monotone and exact over a sample of values (all of them for a short range)
    auto exact = [&](u64 rel) {
        const u64 x = rel >> ii.wshift, s = x >> ii.segshift;
        const u128 g = (u128)tab[s].G + (u128)(x - (s << ii.segshift)) * tab[s].slope;
        const u64 k = (u64)(g >> 32);
        return (u32)(k < ii.nb ? k : ii.nb - 1);
    };
    u32 prev = 0;
    const u64 n = range < 50000 ? range + 1 : 50000;
    for (u64 i = 0; i < n; ++i) {
        const u64 rel = range < 50000 ? i : (u64)((u128)range * i / (n - 1));
        const u32 k = fine_bin(rel, ii, tab);
        ++checks;
        if (k != exact(rel) || k < prev || k >= ii.nb) FAIL("fine_bin: range %llu bins %d kind %d value %llu bin %u exact %u prev %u", range, bins, kind, rel, k, exact(rel), prev);
        prev = k;
    }
}

static void check_fine()
{
    std::vector<u64> ranges = {0, 1, 2, 63, 64, 65, 127, 128, 1000, 4095, 4096, 99999, 1u << 20, 0xffffffffull, 0x100000000ull,
                               0x100000001ull, 123456789012ull, 1ull << 40, (1ull << 52) + 7, (1ull << 62) - 1, 1ull << 62};
    for (int i = 0; i < 60; ++i) ranges.push_back(rnd() >> (rnd() % 62));
    const int binss[] = {2, 3, 17, 512, 4096, 65536, 1 << 20};
    for (u64 range : ranges)
        for (int bins : binss)
            for (int kind = 0; kind < 5; ++kind) fine_case(range, bins, kind);
}

// Division by a remembered reciprocal (the predicted rows' partition kernel divides by every row's interval
// once per fine bin): exact for every numerator, divisors from 2 to 2^32 - 1; 0 and 1 and wider divisors get
// no reciprocal.
static void check_reciprocal()
{
    std::vector<u32> ds = {2u, 3u, 4u, 5u, 7u, 255u, 256u, 257u, 65535u, 65536u, 65537u, 0x7fffffffu, 0x80000000u,
                           0x80000001u, 0xfffffffeu, 0xffffffffu};
    for (int i = 0; i < 3000; ++i) ds.push_back((u32)(rnd() >> (32 + rnd() % 31)) | 2u);
    for (u32 d : ds) {
        const u32 m = row_reciprocal(d);
        std::vector<u32> ns = {0u, 1u, d - 1u, d, d + 1u, 2u * d - 1u, 2u * d, 0x7fffffffu, 0x80000000u, 0xfffffffeu, 0xffffffffu,
                               0xffffffffu / d * d, 0xffffffffu / d * d - 1u};
        for (int i = 0; i < 400; ++i) ns.push_back((u32)rnd());
        for (int i = 0; i < 100; ++i) ns.push_back((u32)(rnd() % 64) * d + (u32)(rnd() % 3) - 1u);     // around multiples of d
        for (u32 n : ns) {
            ++checks;
            if (m == 0 || div_by_reciprocal(n, d, m) != n / d) {
                if (++failures < 20) std::printf("reciprocal: n=%u d=%u m=%u gives %u, want %u\n", n, d, m, m ? div_by_reciprocal(n, d, m) : 0u, n / d);
            }
        }
    }
    ++checks;
    if (row_reciprocal(0) != 0u || row_reciprocal(1) != 0u || row_reciprocal(1ull << 32) != 0u || row_reciprocal(~0ull) != 0u) {
        ++failures;
        std::printf("reciprocal: a divisor without one got one\n");
    }
}

int main()
{
    check_reciprocal();
    std::printf("reciprocals: %lld checks, %lld failures so far\n", checks, failures);
    check_linear();
    std::printf("linear maps: %lld checks, %lld failures so far\n", checks, failures);
    check_table();
    std::printf("table maps: %lld checks, %lld failures so far\n", checks, failures);
    check_fine();
    std::printf("fine-bin grid: %lld checks, %lld failures\n", checks, failures);
    return failures ? 1 : 0;
}

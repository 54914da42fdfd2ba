// Small min/max networks on 32-bit keys held in registers (compare-exchange = v_min_u32 + v_max_u32).
#pragma once
#include "tmask_device.hpp"

namespace tmask {

__device__ __forceinline__ void cmpx(uint32_t &a, uint32_t &b)
{
    const uint32_t lo = a < b ? a : b;
    const uint32_t hi = a < b ? b : a;
    a = lo;
    b = hi;
}

template <int N>
__device__ __forceinline__ void sort_asc(uint32_t (&v)[N]);

// three-input minimum / median / maximum: one instruction each
__device__ __forceinline__ uint32_t min3u(uint32_t a, uint32_t b, uint32_t c)
{
    uint32_t r;
    asm("v_min3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

__device__ __forceinline__ uint32_t max3u(uint32_t a, uint32_t b, uint32_t c)
{
    uint32_t r;
    asm("v_max3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

__device__ __forceinline__ uint32_t med3u(uint32_t a, uint32_t b, uint32_t c)
{
    uint32_t r;
    asm("v_med3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// sorts three keys in place: three instructions for the work of three compare-exchanges (six instructions)
__device__ __forceinline__ void sort3(uint32_t &a, uint32_t &b, uint32_t &c)
{
    const uint32_t lo = min3u(a, b, c), mid = med3u(a, b, c), hi = max3u(a, b, c);
    a = lo;
    b = mid;
    c = hi;
}

template <>
__device__ __forceinline__ void sort_asc<2>(uint32_t (&v)[2])
{
    cmpx(v[0], v[1]);
}

// Four keys: sort the first three, then the last three.  v[3] is then the maximum and v[1] <= v[2]; v[2], the median
// of the old v[1], v[2], v[3], is at least the old v[1] (two of the three are) and so at least v[0]: only v[0] and v[1]
// can still be out of order.  8 instructions against 10 for five compare-exchanges.
template <>
__device__ __forceinline__ void sort_asc<4>(uint32_t (&v)[4])
{
    sort3(v[0], v[1], v[2]); sort3(v[1], v[2], v[3]); cmpx(v[0], v[1]);
}

// Eight keys by eight three-key sorts: 24 instructions against 38 for the best network of compare-exchanges (19).  The
// sequence was found by a search over networks of three-key sorts and compare-exchanges and checked on all 256
// zero-one inputs (a network of sorters sorts every input if it sorts those).
template <>
__device__ __forceinline__ void sort_asc<8>(uint32_t (&v)[8])
{
    sort3(v[4], v[5], v[6]); sort3(v[1], v[2], v[3]); sort3(v[0], v[3], v[7]); sort3(v[0], v[1], v[4]);
    sort3(v[2], v[3], v[5]); sort3(v[5], v[6], v[7]); sort3(v[3], v[4], v[5]); sort3(v[1], v[2], v[3]);
}

// v[0..8) and v[8..16), each ascending -> all of v ascending: thirteen three-key sorts and two compare-exchanges (43
// instructions; Batcher's odd-even merge of two runs of eight takes 25 compare-exchanges, 50 instructions).
__device__ __forceinline__ void merge_sorted8_asc(uint32_t (&v)[16])
{
    sort3(v[0], v[4], v[12]); sort3(v[1], v[5], v[13]); sort3(v[2], v[6], v[14]); sort3(v[7], v[14], v[15]);
    sort3(v[3], v[7], v[11]); sort3(v[2], v[6], v[10]); sort3(v[1], v[5], v[9]); sort3(v[4], v[6], v[8]);
    sort3(v[0], v[2], v[4]); sort3(v[3], v[5], v[6]); sort3(v[7], v[8], v[9]); sort3(v[9], v[10], v[12]);
    sort3(v[11], v[12], v[13]); cmpx(v[3], v[4]); cmpx(v[1], v[2]);
}

// Sixteen keys: both halves by sort_asc<8>, then a merge of two sorted runs of eight out of thirteen three-key sorts and
// two compare-exchanges (found and checked the same way, on the 81 zero-one inputs with sorted halves): 91 instructions
// against 126 for Batcher's odd-even merge sort.
template <>
__device__ __forceinline__ void sort_asc<16>(uint32_t (&v)[16])
{
    uint32_t a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; i++) {
        a[i] = v[i];
        b[i] = v[8 + i];
    }
    sort_asc<8>(a);
    sort_asc<8>(b);
#pragma unroll
    for (int i = 0; i < 8; i++) {
        v[i] = a[i];
        v[8 + i] = b[i];
    }
    merge_sorted8_asc(v);
}

// v[0..N/2) ascending followed by v[N/2..N) descending (a bitonic sequence) -> all of v ascending: log2 N rounds of
// N/2 compare-exchanges at distance N/2, N/4, ..., 1
template <int N>
__device__ __forceinline__ void bitonic_merge_asc(uint32_t (&v)[N])
{
#pragma unroll
    for (int k = N / 2; k >= 1; k /= 2)
#pragma unroll
        for (int i = 0; i < N; i++)
            if ((i & k) == 0)
                cmpx(v[i], v[i + k]);
}

// (H)-th largest of the 2H distinct keys lo[0..H) u hi[0..H): both halves get sorted in place.
template <int H>
__device__ __forceinline__ uint32_t upper_half_min(uint32_t (&a)[H], uint32_t (&b)[H])
{
    sort_asc<H>(a);
    sort_asc<H>(b);
    uint32_t t = 0xFFFFFFFFu;
#pragma unroll
    for (int i = 0; i < H; i++) {
        const uint32_t m = a[i] > b[H - 1 - i] ? a[i] : b[H - 1 - i];
        t = m < t ? m : t;
    }
    return t;
}

// ---- eight values: order statistics from three-input instructions ----------------------------------------------
// The median of nine values laid out 3 x 3 is med3(max of the column minima, med3 of the column medians, min of the
// column maxima).  With +inf as the ninth value that median is the 5th smallest of the other eight, with 0 it is
// their 4th smallest; the two share the column sorts.  12 instructions for one of them, 16 for both, against 27 and
// 36 with two sorted halves.  Values may repeat (order statistics of a multiset).

struct Eight {
    uint32_t l0, m0, h0, l1, m1, h1, l2, h2;   // sorted (v0,v1,v2), sorted (v3,v4,v5), min and max of (v6,v7)
};

__device__ __forceinline__ Eight columns_of_8(const uint32_t (&v)[8])
{
    Eight e;
    e.l0 = min3u(v[0], v[1], v[2]); e.m0 = med3u(v[0], v[1], v[2]); e.h0 = max3u(v[0], v[1], v[2]);
    e.l1 = min3u(v[3], v[4], v[5]); e.m1 = med3u(v[3], v[4], v[5]); e.h1 = max3u(v[3], v[4], v[5]);
    e.l2 = v[6] < v[7] ? v[6] : v[7];
    e.h2 = v[6] < v[7] ? v[7] : v[6];
    return e;
}

// 5th smallest of eight (the smallest of their upper half): ninth value +inf, whose column is (l2, h2, inf)
__device__ __forceinline__ uint32_t fifth_of_8(const Eight &e)
{
    const uint32_t hh = e.h0 < e.h1 ? e.h0 : e.h1;
    return med3u(max3u(e.l0, e.l1, e.l2), med3u(e.m0, e.m1, e.h2), hh);
}

// 4th smallest of eight (the largest of their lower half): ninth value 0, whose column is (0, l2, h2)
__device__ __forceinline__ uint32_t fourth_of_8(const Eight &e)
{
    const uint32_t ll = e.l0 > e.l1 ? e.l0 : e.l1;
    return med3u(ll, med3u(e.m0, e.m1, e.l2), min3u(e.h0, e.h1, e.h2));
}

template <>
__device__ __forceinline__ uint32_t upper_half_min<4>(uint32_t (&a)[4], uint32_t (&b)[4])
{
    const uint32_t v[8] = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
    return fifth_of_8(columns_of_8(v));
}

}  // namespace tmask

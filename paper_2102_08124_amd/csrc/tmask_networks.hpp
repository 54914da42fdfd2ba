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

template <>
__device__ __forceinline__ void sort_asc<2>(uint32_t (&v)[2])
{
    cmpx(v[0], v[1]);
}

template <>
__device__ __forceinline__ void sort_asc<4>(uint32_t (&v)[4])
{
    cmpx(v[0], v[1]); cmpx(v[2], v[3]); cmpx(v[0], v[2]); cmpx(v[1], v[3]); cmpx(v[1], v[2]);
}

template <>
__device__ __forceinline__ void sort_asc<8>(uint32_t (&v)[8])
{
    cmpx(v[0], v[1]); cmpx(v[2], v[3]); cmpx(v[4], v[5]); cmpx(v[6], v[7]);
    cmpx(v[0], v[2]); cmpx(v[1], v[3]); cmpx(v[4], v[6]); cmpx(v[5], v[7]);
    cmpx(v[1], v[2]); cmpx(v[5], v[6]);
    cmpx(v[0], v[4]); cmpx(v[1], v[5]); cmpx(v[2], v[6]); cmpx(v[3], v[7]);
    cmpx(v[2], v[4]); cmpx(v[3], v[5]);
    cmpx(v[1], v[2]); cmpx(v[3], v[4]); cmpx(v[5], v[6]);
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

}  // namespace tmask

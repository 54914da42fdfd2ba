// Algorithm 1 (arXiv 2102.08124, Sec. 4) specialised to M = 4, K = 2: the 2:4 transposable case.
//
// In rank form an entry is kept iff at least K = 2 of the 3 other entries of its row precede it in
// the (magnitude, index) order, and the same in its column.  With p_ab = "position a precedes
// position b" = (key_a <= key_b) for a < b, "at least 2 of 3" is a majority:
//     keep_0 = !maj(p01, p02, p03)      keep_1 = maj(p01, !p12, !p13)
//     keep_2 =  maj(p02, p12, !p23)     keep_3 = maj(p03,  p13,  p23)
// The six compares of a line are vector compares whose results are wavefront lane masks; the
// majority logic then runs on lane masks in the scalar ALU, which issues beside the vector ALU.
#pragma once
#include "tmask_device.hpp"

namespace tmask {

// keep masks of one line of four keys given in position order
__device__ __forceinline__ void top2_of_4(uint32_t k0, uint32_t k1, uint32_t k2, uint32_t k3, lanemask_t &e0,
                                          lanemask_t &e1, lanemask_t &e2, lanemask_t &e3)
{
    const lanemask_t p01 = lm(k0 <= k1), p02 = lm(k0 <= k2), p03 = lm(k0 <= k3);
    const lanemask_t p12 = lm(k1 <= k2), p13 = lm(k1 <= k3), p23 = lm(k2 <= k3);
    e0 = ~maj3(p01, p02, p03);
    e1 = maj3(p01, ~p12, ~p13);
    e2 = maj3(p02, p12, ~p23);
    e3 = maj3(p03, p13, p23);
}

// One 4x4 block: k[i][c] = keys.  Returns the kept magnitudes' sum and writes the keep flags of
// row i as four 0/1 bytes into rowbytes[i].  Column masks are formed first (16 lane masks), rows
// are then finished one at a time so that few lane masks are live at once.
__device__ __forceinline__ float approx_2of4_block(const uint32_t (&k)[4][4], uint32_t (&rowbytes)[4])
{
    lanemask_t ck[4][4];
#pragma unroll
    for (int c = 0; c < 4; c++)
        top2_of_4(k[0][c], k[1][c], k[2][c], k[3][c], ck[0][c], ck[1][c], ck[2][c], ck[3][c]);
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        lanemask_t rk[4];
        top2_of_4(k[i][0], k[i][1], k[i][2], k[i][3], rk[0], rk[1], rk[2], rk[3]);
        uint32_t bytes = 0;
#pragma unroll
        for (int c = 0; c < 4; c++) {
            const bool keep = lm_test(rk[c] & ck[i][c]);
            bytes |= keep ? (1u << (8 * c)) : 0u;
            sum += keep ? __uint_as_float(k[i][c]) : 0.f;
        }
        rowbytes[i] = bytes;
    }
    return sum;
}

// The lane's strip (C = 4: one block, C = 8: two blocks side by side): mask out, kept sum back.
template <int DT, int FMT>
__device__ __forceinline__ float approx_2of4_strip(const MatDev &md, StripPos p, const uint32_t (&a)[4][Geo<DT, 4>::C])
{
    constexpr int C = Geo<DT, 4>::C;
    uint32_t bytes[C / 4][4];
    float sum = 0.f;
#pragma unroll
    for (int b = 0; b < C / 4; b++) {
        uint32_t k[4][4];
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
            for (int c = 0; c < 4; c++)
                k[i][c] = a[i][4 * b + c];
        sum += approx_2of4_block(k, bytes[b]);
    }
    if constexpr (FMT == kMaskU8) {
        char *base = (char *)md.mask + (size_t)p.br * 4 * md.mask_ld + (size_t)p.sc * C;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            if constexpr (C == 4) {
                stream_store(bytes[0][i], (uint32_t *)(base + (size_t)i * md.mask_ld));
            } else {
                u32x2 v;
                v.x = bytes[0][i];
                v.y = bytes[1][i];
                stream_store(v, (u32x2 *)(base + (size_t)i * md.mask_ld));
            }
        }
    } else {
        uint32_t bits[4];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            bits[i] = bytes4_to_bits(bytes[0][i]);
            if constexpr (C == 8)
                bits[i] |= bytes4_to_bits(bytes[1][i]) << 4;
        }
        store_mask<DT, 4, kMaskBits>(md, p, bits);
    }
    return sum;
}

}  // namespace tmask

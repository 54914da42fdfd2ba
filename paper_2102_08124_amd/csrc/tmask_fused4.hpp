// tmask_approx_pack for M = 4, N = 2: Algorithm 1 (arXiv 2102.08124, Sec. 4) and the compression of
// W and W^T in one pass over W.  The mask never travels through memory between the two steps; it is
// written only if the caller wants it.
//
// Same tiling as pack24_kernel (S strips x 4096 / S rows per workgroup, a lane holds whole 4x4 blocks), so
// the keep flags that Algorithm 1's rank form yields as lane masks (tmask_approx4.hpp) feed the slot
// logic of the compaction (tmask_pack4.hpp) directly.
#pragma once
#include <type_traits>

#include "tmask_approx4.hpp"
#include "tmask_device.hpp"
#include "tmask_pack.hpp"
#include "tmask_pack4.hpp"

namespace tmask {

template <int DT, int FMT, bool WMASK, int S>
__global__ __launch_bounds__(kThreads) void approx_pack24_kernel(const FusedArgs args)
{
    using PG = Pack4Geo<DT, S>;
    constexpr int ES = PG::ES, C = PG::C, NG = PG::NG, TR = PG::TR, TC = PG::TC, OTD = PG::OTD, TCP = PG::TCP,
                  IDXB = PG::IDXB, IDXTB = PG::IDXTB, LPR = PG::LPR;

    __shared__ __attribute__((aligned(16))) uint32_t OT[OTD][TCP];      // [position down the column][column]
    __shared__ __attribute__((aligned(16))) uint8_t IDXT[IDXTB][TC];
    __shared__ __attribute__((aligned(16))) uint8_t IDX[TR][IDXB];
    // the four doubles of the objective's workgroup sum reuse the first bytes of IDX once the tile is written out

    const uint32_t tile = blockIdx.x;
    const PackDev d = args.d[find_pack_desc(args, tile)];
    const uint32_t tl = tile - d.tile0;
    uint32_t ty, tx;
    tile_coords(tl, d.tiles_x, (d.rows + TR - 1) / TR, kPackRunRows / TR, ty, tx);
    const uint32_t row0 = ty * TR, col0 = tx * TC;
    const uint32_t tid = threadIdx.x, l = tid & 63u;
    // the wavefront number as a scalar: row addresses below are then scalar too, and a lane adds only
    // its fixed offsets (its strip inside the run, the distance of its sub-row)
    const uint32_t w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t strip = l % (uint32_t)S, sub = l / (uint32_t)S;
    const uint32_t q4 = w * LPR + sub;                 // this lane's run of four block-rows inside the tile
    const uint32_t tcol = strip * C;                   // first column of the lane inside the tile
    const uint32_t col = col0 + tcol;
    const bool strip_ok = col < d.cols;
    const size_t pitchW = (size_t)(d.cols / 4) * 2;    // elements per row of vals
    const size_t lane_w = (size_t)sub * 16u * d.ld * ES + strip * 16u;
    const size_t lane_v = (size_t)sub * 16u * pitchW * ES + strip * 8u;
    const size_t lane_m = (size_t)sub * 16u * d.mask_ld;
    float acc = 0.f;

    // Tiles wholly inside the matrix run a copy of the loop without bounds tests (no branch splits it).
    auto compute = [&](auto edge_tag) {
        constexpr bool EDGE = decltype(edge_tag)::value;
        uint32_t tnib[C];
#pragma unroll
        for (int c = 0; c < C; c++)
            tnib[c] = 0;

        // loads run one block-row ahead of the work on them
        u32x4 rawb[2][4];
        auto issue = [&](int q, u32x4 (&raw)[4]) {
            const uint32_t wrow = row0 + 16u * LPR * w + 4u * (uint32_t)q;    // scalar: the row of sub-row 0
            const uint32_t row = wrow + 16u * sub;
#pragma unroll
            for (int i = 0; i < 4; i++)
                raw[i] = u32x4{0u, 0u, 0u, 0u};
            if (!EDGE || (strip_ok && row < d.rows)) {
#pragma unroll
                for (int i = 0; i < 4; i++)
                    raw[i] = __builtin_nontemporal_load(
                        (const u32x4 *)((const char *)d.w + ((size_t)(wrow + i) * d.ld + col0) * ES + lane_w));
            }
        };
        issue(0, rawb[0]);

#pragma unroll
        for (int q = 0; q < 4; q++) {
            const uint32_t brl = 4 * q4 + q;                       // block-row inside the tile
            const uint32_t wrow = row0 + 16u * LPR * w + 4u * (uint32_t)q;
            const uint32_t row = wrow + 16u * sub;
            const bool ok = !EDGE || (strip_ok && row < d.rows);
            if (q + 1 < 4)
                issue(q + 1, rawb[(q + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            u32x4(&raw)[4] = rawb[q & 1];
            uint32_t rowout[4][2];
            uint32_t rownib[4] = {0u, 0u, 0u, 0u};
            uint32_t rowmask[4][NG];   // U8: four 0/1 bytes per group; BITS: four bits per group
#pragma unroll
            for (int g = 0; g < NG; g++) {
                uint32_t e[4][4], k[4][4];
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const uint32_t dw[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};
#pragma unroll
                    for (int c = 0; c < 4; c++) {
                        if constexpr (DT == kF32) {
                            e[i][c] = dw[c];
                            k[i][c] = dw[c] & 0x7FFFFFFFu;
                        } else {
                            e[i][c] = (c & 1) ? (dw[2 * g + c / 2] >> 16) : (dw[2 * g + c / 2] & 0xFFFFu);
                            k[i][c] = e[i][c] & 0x7FFFu;
                        }
                    }
                }
                // Algorithm 1 in rank form: kept iff among the two heaviest of its row and of its column
                lanemask_t keep[4][4];
#pragma unroll
                for (int c = 0; c < 4; c++)
                    top2_of_4(k[0][c], k[1][c], k[2][c], k[3][c], keep[0][c], keep[1][c], keep[2][c], keep[3][c]);
                __builtin_amdgcn_sched_barrier(0);
                // rows: finish the keep flags, then compress W along the row
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    lanemask_t rk[4];
                    top2_of_4(k[i][0], k[i][1], k[i][2], k[i][3], rk[0], rk[1], rk[2], rk[3]);
                    uint32_t mbits = 0;
#pragma unroll
                    for (int c = 0; c < 4; c++) {
                        keep[i][c] &= rk[c];
                        const uint32_t magf = (DT == kF32) ? k[i][c] : (k[i][c] << 16);
                        acc += __uint_as_float(lm_select(keep[i][c], magf, 0u));   // lanes outside the matrix hold zeros
                        if constexpr (WMASK)
                            mbits |= lm_select(keep[i][c], (FMT == kMaskU8) ? (1u << (8 * c)) : (1u << c), 0u);
                    }
                    // pin the running sum here: left alone, the compiler defers all 64 additions to the end of
                    // the tile and keeps every addend in a register until then.  The same holds for the merges
                    // of position nibbles and mask bits below; those are pinned at bf16 only, where the
                    // registers would otherwise run out (at fp32 the freer schedule is the faster one)
                    asm volatile("" : "+v"(acc));
                    rowmask[i][g] = mbits;
                    if constexpr (WMASK)
                        asm volatile("" : "+v"(rowmask[i][g]));
                    uint32_t v0, v1, nib;
                    compact_2of4(keep[i][0], keep[i][1], keep[i][2], keep[i][3], e[i][0], e[i][1], e[i][2], e[i][3],
                                 v0, v1, nib);
                    if constexpr (DT == kF32) {
                        rowout[i][0] = v0;
                        rowout[i][1] = v1;
                    } else {
                        rowout[i][g] = v0 | (v1 << 16);
                    }
                    rownib[i] |= nib << (4 * g);
                    if constexpr (DT == kBF16)
                        asm volatile("" : "+v"(rownib[i]));
                    __builtin_amdgcn_sched_barrier(0);
                }
                // columns: compress W^T down the column; the slots of the four columns go straight to LDS
                uint32_t t0[4], t1[4];
#pragma unroll
                for (int c = 0; c < 4; c++) {
                    uint32_t nib;
                    compact_2of4(keep[0][c], keep[1][c], keep[2][c], keep[3][c], e[0][c], e[1][c], e[2][c], e[3][c],
                                 t0[c], t1[c], nib);
                    tnib[4 * g + c] |= nib << (4 * q);
                    if constexpr (DT == kBF16) {
                        t0[c] |= t1[c] << 16;
                        asm volatile("" : "+v"(tnib[4 * g + c]));   // merge now, as for the sum above
                        asm volatile("" : "+v"(t0[c]));
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                if constexpr (DT == kF32) {
                    *(u32x4 *)&OT[brl * 2][ot_col(brl * 2, tcol)] = u32x4{t0[0], t0[1], t0[2], t0[3]};
                    *(u32x4 *)&OT[brl * 2 + 1][ot_col(brl * 2 + 1, tcol)] = u32x4{t1[0], t1[1], t1[2], t1[3]};
                } else {
                    *(u32x4 *)&OT[brl][ot_col(brl, tcol + 4 * g)] = u32x4{t0[0], t0[1], t0[2], t0[3]};
                }
            }
            if (EDGE && !ok) {
#pragma unroll
                for (int i = 0; i < 4; i++)
                    rownib[i] = 0;   // nothing of this strip may show up in a row's padding bits
            }
            if constexpr (WMASK && FMT == kMaskBits && C == 4) {
                // two lanes share a mask byte: the even one writes it (exchange outside the bounds test)
#pragma unroll
                for (int i = 0; i < 4; i++)
                    rowmask[i][0] |= quad_xor<1>(rowmask[i][0]) << 4;
            }
            if (ok) {
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    u32x2 v;
                    v.x = rowout[i][0];
                    v.y = rowout[i][1];
                    stream_store(
                        v, (u32x2 *)((char *)d.vals + ((size_t)(wrow + i) * pitchW + (size_t)(col0 / 4) * 2) * ES + lane_v));
                    if constexpr (WMASK) {
                        char *mrow = (char *)const_cast<void *>(d.mask) + (size_t)(wrow + i) * d.mask_ld + lane_m +
                                     ((FMT == kMaskU8) ? col0 : (col0 >> 3));
                        const uint32_t lcol = tcol;              // the lane's first column inside the tile
                        if constexpr (FMT == kMaskU8) {
                            if constexpr (C == 4) {
                                stream_store(rowmask[i][0], (uint32_t *)(mrow + lcol));
                            } else {
                                u32x2 mv;
                                mv.x = rowmask[i][0];
                                mv.y = rowmask[i][NG - 1];
                                stream_store(mv, (u32x2 *)(mrow + lcol));
                            }
                        } else {
                            if constexpr (C == 8) {
                                mrow[lcol >> 3] = (char)(rowmask[i][0] | (rowmask[i][NG - 1] << 4));
                            } else {
                                if ((l & 1u) == 0)
                                    mrow[lcol >> 3] = (char)rowmask[i][0];
                            }
                        }
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < 4; i++) {
                if constexpr (C == 4) {
                    const uint32_t other = quad_xor<1>(rownib[i]);
                    if ((l & 1u) == 0)
                        IDX[4 * brl + i][strip >> 1] = (uint8_t)(rownib[i] | (other << 4));
                } else {
                    IDX[4 * brl + i][strip] = (uint8_t)rownib[i];
                }
            }
        }
        if (EDGE && !strip_ok) {
#pragma unroll
            for (int c = 0; c < C; c++)
                tnib[c] = 0;
        }
        // block-rows of this wavefront that lie outside the matrix must not leave position bits either
        if (EDGE) {
            const uint32_t brs_in = (d.rows - row0) / 4;           // block-rows of the tile inside the matrix
            const uint32_t mine = brs_in > 4 * q4 ? brs_in - 4 * q4 : 0;
            const uint32_t keepmask = mine >= 4 ? 0xFFFFu : ((1u << (4 * mine)) - 1u);
#pragma unroll
            for (int c = 0; c < C; c++)
                tnib[c] &= keepmask;
        }
        // a lane's four nibbles per column are two bytes: two rows of C bytes each
#pragma unroll
        for (int t = 0; t < 2; t++) {
            uint32_t b[C / 4];
#pragma unroll
            for (int h = 0; h < C / 4; h++)
                b[h] = ((tnib[4 * h] >> (8 * t)) & 0xFFu) | (((tnib[4 * h + 1] >> (8 * t)) & 0xFFu) << 8) |
                       (((tnib[4 * h + 2] >> (8 * t)) & 0xFFu) << 16) | (((tnib[4 * h + 3] >> (8 * t)) & 0xFFu) << 24);
            if constexpr (C == 4) {
                *(uint32_t *)&IDXT[2 * q4 + t][tcol] = b[0];
            } else {
                u32x2 v;
                v.x = b[0];
                v.y = b[1];
                *(u32x2 *)&IDXT[2 * q4 + t][tcol] = v;
            }
        }
    };
    if (row0 + TR <= d.rows && col0 + TC <= d.cols)
        compute(std::false_type{});
    else
        compute(std::true_type{});
    __syncthreads();
    pack24_copy_out<DT, S>(d, row0, col0, OT, IDXT, IDX);
    if (args.partials) {
        __syncthreads();                                   // every wavefront is done reading IDX
        double *red = (double *)&IDX[0][0];
        const double t = block_sum_f32(acc, red);
        if (threadIdx.x == 0)
            ((double *)args.partials)[args.partial0 + tile] = t;
    }
}

}  // namespace tmask

// tmask_apply_pack specialised to M = 4, N = 2 (the 2:4 transposable case); same output format as
// the general kernel in tmask_pack.hpp (described in include/tmask.h).
//
// One workgroup packs 64 rows x 64 strips (256 fp32 / 512 bf16 columns).  Wavefront w owns block-rows
// 4w..4w+3 of the tile, lane l owns strip l, so every load is a contiguous 1 KiB run.  A lane holds
// whole groups in both directions (4 columns of a row, 4 rows of a column), so compaction needs no
// exchange: the slot logic runs on lane masks in the scalar ALU and picks values with selects.
//   W   : N values per group go straight from registers to memory (8 B per lane and row);
//         position nibbles are collected per row in LDS and written as whole rows of bytes.
//   W^T : a lane gathers, per column, the 8 values of its four block-rows in registers, parks them in
//         LDS ([column][block-row]) and the workgroup streams 128 B (fp32) / 64 B (bf16) runs per column.
#pragma once
#include <type_traits>

#include "tmask_device.hpp"
#include "tmask_pack.hpp"

namespace tmask {

constexpr int kPack4Rows = 64;     // tile rows
constexpr int kPack4Strips = 64;   // tile strips (16 bytes each)

// r = lane-mask bit set ? a : b, as exactly one v_cndmask with the mask in a scalar register pair
// (written as an instruction because the compiler otherwise turns chains of such selects into
// branches and moves the mask logic into vector registers).
__device__ __forceinline__ uint32_t lm_select(lanemask_t m, uint32_t a, uint32_t b)
{
    uint32_t r;
    asm("v_cndmask_b32_e64 %0, %1, %2, %3" : "=v"(r) : "v"(b), "v"(a), "s"(m));
    return r;
}

// One group of four: k = keep flags (lane masks), e = element bits.  Exactly two slots come out,
// in position order: kept entries (at most the first two), else the lowest unused positions as +0.
__device__ __forceinline__ void compact_2of4(lanemask_t k0, lanemask_t k1, lanemask_t k2, lanemask_t k3, uint32_t e0,
                                             uint32_t e1, uint32_t e2, uint32_t e3, uint32_t &v0, uint32_t &v1,
                                             uint32_t &nibble)
{
    const lanemask_t m012 = maj3(k0, k1, k2);
    const lanemask_t s2 = k2 & ~(k0 & k1), s3 = k3 & ~m012;       // kept beyond the second are dropped
    const lanemask_t ge2 = m012 | (k3 & (k0 | k1 | k2));
    const lanemask_t any = k0 | k1 | k2 | k3;
    const lanemask_t c0 = k0 | ~ge2;
    const lanemask_t c1 = k1 | (~ge2 & (k0 | ~any));
    // slot 0 holds position 0 if chosen, else 1 if chosen, else 2; its value is non-zero only for kept entries
    v0 = lm_select(k0, e0, lm_select(c0, 0u, lm_select(k1, e1, lm_select(c1, 0u, lm_select(s2, e2, 0u)))));
    // slot 1 holds position 3 if kept, else 2 if kept, else 1 (kept or filler)
    v1 = lm_select(s3, e3, lm_select(s2, e2, lm_select(k1, e1, 0u)));
    // positions: slot0 = c0 ? 0 : c1 ? 1 : 2, slot1 = s3 ? 3 : s2 ? 2 : 1
    nibble = lm_select(~c0 & c1, 1u, 0u) | lm_select(~c0 & ~c1, 2u, 0u) | lm_select(s3 | ~s2, 4u, 0u) |
             lm_select(s3 | s2, 8u, 0u);
}

// Keep flag of column c (0..7) of a row as a lane mask. U8: m0/m1 = the row's mask bytes as dwords
// (any non-zero byte = kept); BITS: m0 = the row's mask bits.
template <int FMT>
__device__ __forceinline__ lanemask_t keep_flag(uint32_t m0, uint32_t m1, int c)
{
    if constexpr (FMT == kMaskU8)
        return lm((((c < 4) ? m0 : m1) & (0xFFu << (8 * (c & 3)))) != 0u);
    else
        return lm((m0 & (1u << c)) != 0u);
}

// Tile geometry of the 2:4 pack kernels for one element type.
template <int DT>
struct Pack4Geo {
    static constexpr int ES = (DT == kF32) ? 4 : 2;
    static constexpr int C = 16 / ES;                  // columns per strip
    static constexpr int NG = C / 4;                   // groups per strip row
    static constexpr int TR = kPack4Rows, TS = kPack4Strips, TC = TS * C;
    static constexpr int VPC = (DT == kF32) ? 8 : 4;   // dwords a lane produces per column for W^T (4 block-rows)
    static constexpr int OTD = 4 * VPC;                // data dwords per column in the tile (16 block-rows)
    static constexpr int OTW = OTD + 4;                // padded, keeps 16-byte alignment
    static constexpr int IDXB = TS * NG / 2;           // index bytes per tile row
};

// Streams a finished tile out of LDS: OT = W^T values per column, IDXT = W^T position nibbles per
// column, IDX = W position nibbles per row.  Call after a barrier; all threads take part.
template <int DT>
__device__ __forceinline__ void pack24_copy_out(const PackDev &d, uint32_t row0, uint32_t col0,
                                                const uint32_t (*OT)[Pack4Geo<DT>::OTW], const uint16_t (*IDXT)[4],
                                                const uint8_t (*IDX)[Pack4Geo<DT>::IDXB])
{
    using PG = Pack4Geo<DT>;
    constexpr int ES = PG::ES, TR = PG::TR, TC = PG::TC, OTD = PG::OTD;
    const uint32_t tid = threadIdx.x;
    const size_t pitchT = (size_t)(d.rows / 4) * 2;    // elements per row of valsT
    const uint32_t cols_valid = min((uint32_t)TC, d.cols - col0);
    const uint32_t brs_valid = min((uint32_t)(TR / 4), (d.rows - row0) / 4);
    const uint32_t rows_valid = brs_valid * 4;
    // ---- valsT ----
    {
        char *dst = (char *)d.valsT + ((size_t)col0 * pitchT + (size_t)(row0 / 4) * 2) * ES;
        const size_t pitch_b = pitchT * ES;
        if (brs_valid == TR / 4 && (pitch_b & 15) == 0 && (((uintptr_t)dst) & 15) == 0) {
            constexpr int CH = OTD / 4;   // 16-byte chunks per column
            for (uint32_t j = tid; j < cols_valid * CH; j += kThreads) {
                const uint32_t cc = j / CH, part = j % CH;
                const u32x4 v = *(const u32x4 *)&OT[cc][4 * part];
                __builtin_nontemporal_store(v, (u32x4 *)(dst + (size_t)cc * pitch_b + 16 * part));
            }
        } else {
            const uint32_t rd = brs_valid * 2 * ES / 4;   // dwords per column
            for (uint32_t j = tid; j < cols_valid * rd; j += kThreads) {
                const uint32_t cc = j / rd, x = j - cc * rd;
                *(uint32_t *)(dst + (size_t)cc * pitch_b + 4 * x) = OT[cc][x];
            }
        }
    }
    // ---- idx ----
    {
        const size_t pitch = ((size_t)d.cols + 7) / 8;
        const uint32_t nb = (cols_valid / 4 + 1) / 2;
        unsigned char *dst = (unsigned char *)d.idx + (size_t)row0 * pitch + col0 / 8;
        if ((nb & 3) == 0 && (pitch & 3) == 0 && (((uintptr_t)dst) & 3) == 0) {
            const uint32_t nd = nb / 4;
            for (uint32_t j = tid; j < rows_valid * nd; j += kThreads) {
                const uint32_t r = j / nd, x = j - r * nd;
                *(uint32_t *)(dst + (size_t)r * pitch + 4 * x) = ((const uint32_t *)&IDX[r][0])[x];
            }
        } else {
            for (uint32_t j = tid; j < rows_valid * nb; j += kThreads) {
                const uint32_t r = j / nb, x = j - r * nb;
                dst[(size_t)r * pitch + x] = IDX[r][x];
            }
        }
    }
    // ---- idxT ----
    {
        const size_t pitch = ((size_t)d.rows + 7) / 8;
        const uint32_t nb = (brs_valid + 1) / 2;
        unsigned char *dst = (unsigned char *)d.idxT + (size_t)col0 * pitch + row0 / 8;
        if (nb == 8 && (pitch & 7) == 0 && (((uintptr_t)dst) & 7) == 0) {
            for (uint32_t cc = tid; cc < cols_valid; cc += kThreads)
                *(u32x2 *)(dst + (size_t)cc * pitch) = *(const u32x2 *)&IDXT[cc][0];
        } else {
            for (uint32_t j = tid; j < cols_valid * nb; j += kThreads) {
                const uint32_t cc = j / nb, x = j - cc * nb;
                dst[(size_t)cc * pitch + x] = ((const unsigned char *)&IDXT[cc][0])[x];
            }
        }
    }
}

template <int DT, int FMT>
__global__ __launch_bounds__(kThreads) void pack24_kernel(const PackArgs args)
{
    using PG = Pack4Geo<DT>;
    constexpr int ES = PG::ES, C = PG::C, NG = PG::NG, TR = PG::TR, TC = PG::TC, VPC = PG::VPC, OTW = PG::OTW,
                  IDXB = PG::IDXB;

    __shared__ __attribute__((aligned(16))) uint32_t OT[TC][OTW];
    __shared__ __attribute__((aligned(8))) uint16_t IDXT[TC][4];
    __shared__ __attribute__((aligned(16))) uint8_t IDX[TR][IDXB];

    const uint32_t tile = blockIdx.x;
    int lo = 0, hi = (int)args.n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (args.d[mid].tile0 <= tile)
            lo = mid;
        else
            hi = mid - 1;
    }
    const PackDev d = args.d[lo];
    const uint32_t tl = tile - d.tile0;
    const uint32_t ty = tl / d.tiles_x, tx = tl - ty * d.tiles_x;
    const uint32_t row0 = ty * TR, col0 = tx * TC;
    const uint32_t tid = threadIdx.x, l = tid & 63u;
    // the wavefront number as a scalar: row addresses below are then scalar too, and a lane adds only
    // its fixed offset inside the 1 KiB run
    const uint32_t w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t col = col0 + l * C;
    const bool strip_ok = col < d.cols;
    const size_t pitchW = (size_t)(d.cols / 4) * 2;    // elements per row of vals
    const size_t pitchT = (size_t)(d.rows / 4) * 2;    // elements per row of valsT

    // Tiles that lie wholly inside the matrix take a copy of the code without any bounds test: no branch
    // splits the loop, so the waits on the prefetched rows are exact.
    auto compute = [&](auto edge_tag) {
        constexpr bool EDGE = decltype(edge_tag)::value;
        uint32_t vt[C][VPC];
        uint32_t tnib[C];
#pragma unroll
        for (int c = 0; c < C; c++)
            tnib[c] = 0;

        // Loads run one block-row ahead of the compaction: while block-row q is worked on, the 16-byte rows
        // and mask entries of block-row q + 1 are already in flight.
        u32x4 rawb[2][4];
        uint32_t m0b[2][4], m1b[2][4];   // the rows' mask entries: U8 bytes as dwords, or BITS in m0
        auto issue = [&](int q, u32x4 (&raw)[4], uint32_t (&m0)[4], uint32_t (&m1)[4]) {
            const uint32_t row = row0 + 4 * (4 * w + (uint32_t)q);
#pragma unroll
            for (int i = 0; i < 4; i++) {
                raw[i] = u32x4{0u, 0u, 0u, 0u};
                m0[i] = m1[i] = 0;
            }
            if (!EDGE || (strip_ok && row < d.rows)) {
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    raw[i] = __builtin_nontemporal_load(
                        (const u32x4 *)((const char *)d.w + ((size_t)(row + i) * d.ld + col0) * ES + l * 16u));
                    if constexpr (FMT == kMaskU8) {
                        const char *mp = (const char *)d.mask + ((size_t)(row + i) * d.mask_ld + col0) + l * (uint32_t)C;
                        if constexpr (C == 4) {
                            m0[i] = __builtin_nontemporal_load((const uint32_t *)mp);
                        } else {
                            const u32x2 mv = __builtin_nontemporal_load((const u32x2 *)mp);
                            m0[i] = mv.x;
                            m1[i] = mv.y;
                        }
                    } else {
                        const uint32_t byte = ((const unsigned char *)d.mask)[(size_t)(row + i) * d.mask_ld + (col >> 3)];
                        m0[i] = (C == 8) ? byte : ((byte >> (col & 4u)) & 0xFu);
                    }
                }
            }
        };
        issue(0, rawb[0], m0b[0], m1b[0]);

#pragma unroll
        for (int q = 0; q < 4; q++) {
            const uint32_t brl = 4 * w + q;
            const uint32_t row = row0 + 4 * brl;
            const bool ok = !EDGE || (strip_ok && row < d.rows);
            if (q + 1 < 4)
                issue(q + 1, rawb[(q + 1) & 1], m0b[(q + 1) & 1], m1b[(q + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            u32x4(&raw)[4] = rawb[q & 1];
            uint32_t(&m0)[4] = m0b[q & 1];
            uint32_t(&m1)[4] = m1b[q & 1];
            uint32_t rowout[4][2];
            uint32_t rownib[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int g = 0; g < NG; g++) {
                uint32_t e[4][4];
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const uint32_t dw[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};
#pragma unroll
                    for (int c = 0; c < 4; c++) {
                        if constexpr (DT == kF32)
                            e[i][c] = dw[c];
                        else
                            e[i][c] = (c & 1) ? (dw[2 * g + c / 2] >> 16) : (dw[2 * g + c / 2] & 0xFFFFu);
                    }
                }
                // Lane masks are formed per group right where they are used (and the scheduler is fenced
                // between groups) so that only a handful of them are live at a time.
                // W: groups along the row
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    uint32_t v0, v1, nib;
                    compact_2of4(keep_flag<FMT>(m0[i], m1[i], 4 * g), keep_flag<FMT>(m0[i], m1[i], 4 * g + 1),
                                 keep_flag<FMT>(m0[i], m1[i], 4 * g + 2), keep_flag<FMT>(m0[i], m1[i], 4 * g + 3), e[i][0],
                                 e[i][1], e[i][2], e[i][3], v0, v1, nib);
                    if constexpr (DT == kF32) {
                        rowout[i][0] = v0;
                        rowout[i][1] = v1;
                    } else {
                        rowout[i][g] = v0 | (v1 << 16);
                    }
                    rownib[i] |= nib << (4 * g);
                    __builtin_amdgcn_sched_barrier(0);
                }
                // W^T: groups down the column
#pragma unroll
                for (int c = 0; c < 4; c++) {
                    uint32_t v0, v1, nib;
                    compact_2of4(keep_flag<FMT>(m0[0], m1[0], 4 * g + c), keep_flag<FMT>(m0[1], m1[1], 4 * g + c),
                                 keep_flag<FMT>(m0[2], m1[2], 4 * g + c), keep_flag<FMT>(m0[3], m1[3], 4 * g + c), e[0][c],
                                 e[1][c], e[2][c], e[3][c], v0, v1, nib);
                    if constexpr (DT == kF32) {
                        vt[c][2 * q] = v0;
                        vt[c][2 * q + 1] = v1;
                    } else {
                        vt[4 * g + c][q] = v0 | (v1 << 16);
                    }
                    tnib[4 * g + c] |= nib << (4 * q);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (!ok) {
#pragma unroll
                for (int i = 0; i < 4; i++)
                    rownib[i] = 0;   // nothing of this strip may show up in a row's padding bits
            }
            if (ok) {
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    u32x2 v;
                    v.x = rowout[i][0];
                    v.y = rowout[i][1];
                    __builtin_nontemporal_store(
                        v, (u32x2 *)((char *)d.vals + ((size_t)(row + i) * pitchW + (size_t)(col0 / 4) * 2) * ES + l * 8u));
                }
            }
#pragma unroll
            for (int i = 0; i < 4; i++) {
                if constexpr (C == 4) {
                    const uint32_t other = quad_xor<1>(rownib[i]);
                    if ((l & 1u) == 0)
                        IDX[4 * brl + i][l >> 1] = (uint8_t)(rownib[i] | (other << 4));
                } else {
                    IDX[4 * brl + i][l] = (uint8_t)rownib[i];
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
            const uint32_t mine = brs_in > 4 * w ? brs_in - 4 * w : 0;
            const uint32_t keepmask = mine >= 4 ? 0xFFFFu : ((1u << (4 * mine)) - 1u);
#pragma unroll
            for (int c = 0; c < C; c++)
                tnib[c] &= keepmask;
        }
#pragma unroll
        for (int c = 0; c < C; c++) {
#pragma unroll
            for (int h = 0; h < VPC / 4; h++) {
                u32x4 v = {vt[c][4 * h], vt[c][4 * h + 1], vt[c][4 * h + 2], vt[c][4 * h + 3]};
                *(u32x4 *)&OT[l * C + c][w * VPC + 4 * h] = v;
            }
            IDXT[l * C + c][w] = (uint16_t)tnib[c];
        }
    };
    if (row0 + TR <= d.rows && col0 + TC <= d.cols)
        compute(std::false_type{});
    else
        compute(std::true_type{});
    __syncthreads();

    pack24_copy_out<DT>(d, row0, col0, OT, IDXT, IDX);
}

}  // namespace tmask

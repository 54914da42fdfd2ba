// tmask_apply_pack specialised to M = 4, N = 2 (the 2:4 transposable case); same output format as
// the general kernel in tmask_pack.hpp (described in include/tmask.h).
//
// One workgroup packs a tile of 64 KiB of W: S strips of 16 bytes wide, 4096 / S rows high (Pack4Geo).  A
// wavefront owns 64 / S runs of four block-rows, a lane one strip of one run, so every load is a contiguous
// run of 16 S bytes.  A lane holds
// whole groups in both directions (4 columns of a row, 4 rows of a column), so compaction needs no
// exchange: the slot logic runs on lane masks in the scalar ALU and picks values with selects.
//   W   : N values per group go straight from registers to memory (8 B per lane and row);
//         position nibbles are collected per row in LDS and written as whole rows of bytes.
//   W^T : the two slots of every column group go to LDS as [position down the column][column], written
//         in 16-byte pieces (a lane's columns are neighbours); the workgroup then streams whole runs per column.
#pragma once
#include <type_traits>

#include "tmask_device.hpp"
#include "tmask_pack.hpp"

namespace tmask {

constexpr int kPack4Strips = 64;   // default tile width in strips of 16 bytes
// Fewer resident tiles per compute unit than would fit run faster at fp32 (a tile stays resident for about 20 us
// with four of them, half of a short launch; fewer of them finish sooner and leave a shorter tail, and fewer rows of
// the matrix are open at a time): two for pack24_kernel (41.1 against 42.4 us on the ResNet-50 set, 75 against 72 %
// of the HBM peak on 8192 x 8192), three for the one-pass kernel (37.5 against 40.9 us with two).  The launches ask
// for this much dynamic LDS on top, which nobody uses, so that no further workgroup fits.
constexpr unsigned kPack4LdsReservePackF32 = 18432;
constexpr unsigned kPack4LdsReserveFusedF32 = 8192;

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

// Tile geometry of the 2:4 pack kernels for one element type.  A tile is S strips wide; a wavefront
// covers 64 / S block-rows per step (lane l: strip l % S, sub-row l / S) and takes four steps, so a tile
// has 4096 / S rows: 64 KiB of W whatever S is.  A narrower, taller tile makes the runs written per
// column of W^T longer at the price of shorter runs per row of W.
template <int DT, int S = kPack4Strips, int NW = 4, int QN = 4>
struct Pack4Geo {
    static constexpr int ES = (DT == kF32) ? 4 : 2;
    static constexpr int C = 16 / ES;                  // columns per strip
    static constexpr int NG = C / 4;                   // groups per strip row
    static constexpr int LPR = 64 / S;                 // block-rows a wavefront touches per step
    static constexpr int NT = 64 * NW;                 // threads per workgroup
    static constexpr int TS = S, TR = 4 * QN * LPR * NW, TC = TS * C;   // QN = block-rows a lane works through
    static constexpr int VPB = (DT == kF32) ? 2 : 1;   // dwords per column and block-row for W^T
    static constexpr int OTD = (TR / 4) * VPB;         // data dwords per column in the tile
    static constexpr int TCP = TC;                     // pitch of the staging rows: no padding, see ot_col
    static constexpr int IDXB = TS * NG / 2;           // index bytes per tile row
    static constexpr int IDXTB = TR / 8;               // index bytes per tile column (a nibble per block-row)
};

// Where column `col` of staging row `r` lives: the rows are a whole number of bank cycles long, so the copy-out,
// which reads four consecutive rows of one column per lane, would meet one bank over and over; the column is
// therefore exchanged in units of four (16-byte pieces stay whole) with a pattern that changes every four rows.
// (Padding the rows instead would cost 512 bytes, exactly what keeps a fourth bf16 workgroup off a compute unit.)
__device__ __forceinline__ uint32_t ot_col(uint32_t r, uint32_t col) { return col ^ (((r >> 2) & 7u) << 2); }

// Streams a finished tile out of LDS: OT = W^T values per column, IDXT = W^T position nibbles per
// column, IDX = W position nibbles per row.  Call after a barrier; all threads take part.
template <int DT, int S = kPack4Strips, int NW = 4, int QN = 4>
__device__ __forceinline__ void pack24_copy_out(const PackDev &d, uint32_t row0, uint32_t col0,
                                                const uint32_t (*OT)[Pack4Geo<DT, S, NW, QN>::TCP],
                                                const uint8_t (*IDXT)[Pack4Geo<DT, S, NW, QN>::TC],
                                                const uint8_t (*IDX)[Pack4Geo<DT, S, NW, QN>::IDXB])
{
    using PG = Pack4Geo<DT, S, NW, QN>;
    constexpr uint32_t kNT = PG::NT;
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
            for (uint32_t j = tid; j < cols_valid * CH; j += kNT) {
                const uint32_t cc = j / CH, part = j % CH;
                const uint32_t sc = ot_col(4 * part, cc);          // the same for the four rows 4 part .. 4 part + 3
                const u32x4 v = {OT[4 * part][sc], OT[4 * part + 1][sc], OT[4 * part + 2][sc], OT[4 * part + 3][sc]};
                stream_store(v, (u32x4 *)(dst + (size_t)cc * pitch_b + 16 * part));
            }
        } else {
            const uint32_t rd = brs_valid * 2 * ES / 4;   // dwords per column
            for (uint32_t j = tid; j < cols_valid * rd; j += kNT) {
                const uint32_t cc = j / rd, x = j - cc * rd;
                *(uint32_t *)(dst + (size_t)cc * pitch_b + 4 * x) = OT[x][ot_col(x, cc)];
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
            for (uint32_t j = tid; j < rows_valid * nd; j += kNT) {
                const uint32_t r = j / nd, x = j - r * nd;
                *(uint32_t *)(dst + (size_t)r * pitch + 4 * x) = ((const uint32_t *)&IDX[r][0])[x];
            }
        } else {
            for (uint32_t j = tid; j < rows_valid * nb; j += kNT) {
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
        if (nb == TR / 8 && (pitch & 7) == 0 && (((uintptr_t)dst) & 7) == 0) {
            constexpr uint32_t P = TR / 64;   // 8-byte pieces per column
            for (uint32_t j = tid; j < cols_valid * P; j += kNT) {
                const uint32_t cc = j / P, x = j % P;
                u32x2 v;
                v.x = (uint32_t)IDXT[8 * x][cc] | ((uint32_t)IDXT[8 * x + 1][cc] << 8) |
                      ((uint32_t)IDXT[8 * x + 2][cc] << 16) | ((uint32_t)IDXT[8 * x + 3][cc] << 24);
                v.y = (uint32_t)IDXT[8 * x + 4][cc] | ((uint32_t)IDXT[8 * x + 5][cc] << 8) |
                      ((uint32_t)IDXT[8 * x + 6][cc] << 16) | ((uint32_t)IDXT[8 * x + 7][cc] << 24);
                *(u32x2 *)(dst + (size_t)cc * pitch + 8 * x) = v;
            }
        } else {
            for (uint32_t j = tid; j < cols_valid * nb; j += kNT) {
                const uint32_t cc = j / nb, x = j - cc * nb;
                dst[(size_t)cc * pitch + x] = IDXT[x][cc];
            }
        }
    }
}

template <int DT, int FMT, int S, int NW, int QN>
__global__ __launch_bounds__(64 * NW) void pack24_kernel(const PackArgs args)
{
    static_assert(QN == 2 || QN == 4, "a lane works through two or four block-rows");
    using PG = Pack4Geo<DT, S, NW, QN>;
    constexpr int ES = PG::ES, C = PG::C, NG = PG::NG, TR = PG::TR, TC = PG::TC, OTD = PG::OTD,
                  TCP = PG::TCP, IDXB = PG::IDXB, LPR = PG::LPR, IDXTB = PG::IDXTB;

    // Staging for W^T, indexed [position down the column][column]: a lane's columns are neighbours, so it
    // writes whole 16-byte pieces and the lanes of a wavefront write one contiguous run.
    __shared__ __attribute__((aligned(16))) uint32_t OT[OTD][TCP];
    __shared__ __attribute__((aligned(16))) uint8_t IDXT[IDXTB][TC];
    __shared__ __attribute__((aligned(16))) uint8_t IDX[TR][IDXB];

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
    const uint32_t col = col0 + strip * C;
    const uint32_t tcol = strip * C;                   // first column of the lane inside the tile
    const bool strip_ok = col < d.cols;
    const size_t pitchW = (size_t)(d.cols / 4) * 2;    // elements per row of vals
    // byte offsets of the lane against row 16 * LPR * w of the tile, column col0
    constexpr uint32_t RUN = 4u * QN;                   // rows of a lane's run of block-rows
    const size_t lane_w = (size_t)sub * RUN * d.ld * ES + strip * 16u;
    const size_t lane_m = (size_t)sub * RUN * d.mask_ld;
    const size_t lane_v = (size_t)sub * RUN * pitchW * ES + strip * 8u;

    // Tiles that lie wholly inside the matrix take a copy of the code without any bounds test: no branch
    // splits the loop, so the waits on the prefetched rows are exact.
    auto compute = [&](auto edge_tag) {
        constexpr bool EDGE = decltype(edge_tag)::value;
        uint32_t tnib[C];
#pragma unroll
        for (int c = 0; c < C; c++)
            tnib[c] = 0;

        // Loads run one block-row ahead of the compaction: while block-row q is worked on, the 16-byte rows
        // and mask entries of block-row q + 1 are already in flight.
        constexpr int DEPTH = 2;
        u32x4 rawb[DEPTH][4];
        uint32_t m0b[DEPTH][4], m1b[DEPTH][4];   // the rows' mask entries: U8 bytes as dwords, or BITS in m0
        auto issue = [&](int q, u32x4 (&raw)[4], uint32_t (&m0)[4], uint32_t (&m1)[4]) {
            const uint32_t wrow = row0 + RUN * LPR * w + 4u * (uint32_t)q;    // scalar: the row of sub-row 0
            const uint32_t row = wrow + RUN * sub;
#pragma unroll
            for (int i = 0; i < 4; i++) {
                raw[i] = u32x4{0u, 0u, 0u, 0u};
                m0[i] = m1[i] = 0;
            }
            if (!EDGE || (strip_ok && row < d.rows)) {
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    raw[i] = __builtin_nontemporal_load(
                        (const u32x4 *)((const char *)d.w + ((size_t)(wrow + i) * d.ld + col0) * ES + lane_w));
                    if constexpr (FMT == kMaskU8) {
                        const char *mp = (const char *)d.mask + ((size_t)(wrow + i) * d.mask_ld + col0) + lane_m + tcol;
                        if constexpr (C == 4) {
                            m0[i] = __builtin_nontemporal_load((const uint32_t *)mp);
                        } else {
                            const u32x2 mv = __builtin_nontemporal_load((const u32x2 *)mp);
                            m0[i] = mv.x;
                            m1[i] = mv.y;
                        }
                    } else {
                        const uint32_t byte =
                            ((const unsigned char *)d.mask)[(size_t)(wrow + i) * d.mask_ld + lane_m + (col >> 3)];
                        m0[i] = (C == 8) ? byte : ((byte >> (col & 4u)) & 0xFu);
                    }
                }
            }
        };
#pragma unroll
        for (int q = 0; q < DEPTH - 1; q++)
            issue(q, rawb[q], m0b[q], m1b[q]);

#pragma unroll
        for (int q = 0; q < QN; q++) {
            const uint32_t brl = QN * q4 + q;                      // block-row inside the tile
            const uint32_t wrow = row0 + RUN * LPR * w + 4u * (uint32_t)q;
            const uint32_t row = wrow + RUN * sub;
            const bool ok = !EDGE || (strip_ok && row < d.rows);
            if (q + DEPTH - 1 < QN)
                issue(q + DEPTH - 1, rawb[(q + DEPTH - 1) % DEPTH], m0b[(q + DEPTH - 1) % DEPTH], m1b[(q + DEPTH - 1) % DEPTH]);
            __builtin_amdgcn_sched_barrier(0);
            u32x4(&raw)[4] = rawb[q % DEPTH];
            uint32_t(&m0)[4] = m0b[q % DEPTH];
            uint32_t(&m1)[4] = m1b[q % DEPTH];
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
                    // bf16: without the pins the compiler keeps every select result alive and merges at the end
                    if constexpr (DT == kBF16) {
                        asm volatile("" : "+v"(rownib[i]));
                        asm volatile("" : "+v"(rowout[i][g]));
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                // W^T: groups down the column; the slots of the four columns go straight to LDS
                uint32_t t0[4], t1[4];
#pragma unroll
                for (int c = 0; c < 4; c++) {
                    uint32_t nib;
                    compact_2of4(keep_flag<FMT>(m0[0], m1[0], 4 * g + c), keep_flag<FMT>(m0[1], m1[1], 4 * g + c),
                                 keep_flag<FMT>(m0[2], m1[2], 4 * g + c), keep_flag<FMT>(m0[3], m1[3], 4 * g + c), e[0][c],
                                 e[1][c], e[2][c], e[3][c], t0[c], t1[c], nib);
                    tnib[4 * g + c] |= nib << (4 * q);
                    if constexpr (DT == kBF16) {
                        t0[c] |= t1[c] << 16;
                        asm volatile("" : "+v"(tnib[4 * g + c]));
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
                    stream_store(v, (u32x2 *)((char *)d.vals + ((size_t)(wrow + i) * pitchW + (size_t)(col0 / 4) * 2) * ES + lane_v));
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
        if (EDGE) {
            // strips and block-rows outside the matrix must not leave position bits
            const uint32_t brs_in = (d.rows - row0) / 4;           // block-rows of the tile inside the matrix
            const uint32_t mine = brs_in > QN * q4 ? brs_in - QN * q4 : 0;
            const uint32_t keepmask = !strip_ok ? 0u : mine >= (uint32_t)QN ? 0xFFFFu : ((1u << (4 * mine)) - 1u);
#pragma unroll
            for (int c = 0; c < C; c++)
                tnib[c] &= keepmask;
        }
        // the lane's columns are neighbours here too: its QN nibbles per column are QN / 2 bytes, written as
        // QN / 2 rows of C bytes
#pragma unroll
        for (int t = 0; t < QN / 2; t++) {
            uint32_t b[C / 4];
#pragma unroll
            for (int h = 0; h < C / 4; h++)
                b[h] = ((tnib[4 * h] >> (8 * t)) & 0xFFu) | (((tnib[4 * h + 1] >> (8 * t)) & 0xFFu) << 8) |
                       (((tnib[4 * h + 2] >> (8 * t)) & 0xFFu) << 16) | (((tnib[4 * h + 3] >> (8 * t)) & 0xFFu) << 24);
            if constexpr (C == 4) {
                *(uint32_t *)&IDXT[(QN / 2) * q4 + t][tcol] = b[0];
            } else {
                u32x2 v;
                v.x = b[0];
                v.y = b[1];
                *(u32x2 *)&IDXT[(QN / 2) * q4 + t][tcol] = v;
            }
        }
    };
    if (row0 + TR <= d.rows && col0 + TC <= d.cols)
        compute(std::false_type{});
    else
        compute(std::true_type{});
    __syncthreads();

    pack24_copy_out<DT, S, NW, QN>(d, row0, col0, OT, IDXT, IDX);
}

}  // namespace tmask

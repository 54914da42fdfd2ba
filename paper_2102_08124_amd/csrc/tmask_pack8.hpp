// tmask_apply_pack specialised to bf16, M = 8, N = 4 (the 4:8 transposable case); same output format as
// the general kernel in tmask_pack.hpp (described in include/tmask.h).
//
// A strip of 16 bytes is one group of eight bf16 values, so a lane holds a whole 8 x 8 block per step: its
// eight rows are the row groups, and the same registers read down are the column groups.  A group is
// compacted without loops over slots: the 8-bit set of kept positions indexes a table (built in LDS by
// the workgroup) that holds the byte selectors of four v_perm_b32 and the 12 position bits, so four
// permutes pick the four slots out of the group's four dwords.  Pruned values are zeroed once per block,
// which also makes fillers +0.  Tile = 128 rows x 32 strips (256 columns); a wavefront covers two runs of
// two block-rows per step pair, W values go straight to memory (8 B per lane and row), W^T values and the
// position bits of both directions are staged in LDS and streamed out in whole runs.
#pragma once
#include "tmask_approx_sel.hpp"
#include "tmask_device.hpp"
#include "tmask_pack.hpp"
#include "tmask_pack4.hpp"

namespace tmask {

struct Pack8Geo {
    static constexpr int S = 32;                 // strips per tile row
    static constexpr int LPR = 64 / S;           // runs of block-rows a wavefront covers at a time
    static constexpr int NSTEP = 2;              // block-rows per run
    static constexpr int TR = 4 * LPR * NSTEP * 8, TC = S * 8;
    static constexpr int NBR = TR / 8;           // block-rows per tile
    static constexpr int OTD = NBR * 2;          // dwords per column of W^T in the tile
    static constexpr int TCP = TC + 4;
    static constexpr int IDXB = S * 12 / 8;      // position bytes per tile row
    static constexpr int IDXTB = NBR * 12 / 8;   // position bytes per tile column
};

// the 8 x 8 bit matrix rb (bit c of rb[i] = entry (i, c)) transposed: bit i of the result's byte c
__device__ __forceinline__ void transpose_bits8(const uint32_t (&rb)[8], uint32_t &x, uint32_t &y)
{
    x = rb[0] | (rb[1] << 8) | (rb[2] << 16) | (rb[3] << 24);
    y = rb[4] | (rb[5] << 8) | (rb[6] << 16) | (rb[7] << 24);
    uint32_t t;
    t = (x ^ (x >> 7)) & 0x00AA00AAu;  x ^= t ^ (t << 7);      // 2 x 2 blocks
    t = (y ^ (y >> 7)) & 0x00AA00AAu;  y ^= t ^ (t << 7);
    t = (x ^ (x >> 14)) & 0x0000CCCCu; x ^= t ^ (t << 14);     // 4 x 4 blocks
    t = (y ^ (y >> 14)) & 0x0000CCCCu; y ^= t ^ (t << 14);
    t = (x & 0x0F0F0F0Fu) | ((y << 4) & 0xF0F0F0F0u);          // the two 4 x 4 blocks off the diagonal
    y = ((x >> 4) & 0x0F0F0F0Fu) | (y & 0xF0F0F0F0u);
    x = t;
}

// One group of eight bf16 values given as four dwords (pruned ones already zero): the four slots as two
// dwords, and the 12 position bits.
__device__ __forceinline__ void compact_4of8(uint32_t kbits, uint32_t d0, uint32_t d1, uint32_t d2, uint32_t d3,
                                             const u32x4 *luts, const uint16_t *lutc, uint32_t &o0, uint32_t &o1,
                                             uint32_t &code)
{
    const u32x4 L = luts[kbits];
    code = lutc[kbits];
    o0 = __builtin_amdgcn_perm(d1, d0, L.x) | __builtin_amdgcn_perm(d3, d2, L.y);
    o1 = __builtin_amdgcn_perm(d1, d0, L.z) | __builtin_amdgcn_perm(d3, d2, L.w);
}

// Streams a finished tile out of LDS: OT = W^T values per column, IDXT = W^T position bits per column (bytes),
// IDX = W position bits per row.  Call after a barrier; all NT threads take part.
template <int ES, int TR, int TC, int TCP, int IDXB, int IDXTB, int NT>
__device__ __forceinline__ void pack48_copy_out(const PackDev &d, uint32_t row0, uint32_t col0,
                                                const uint32_t (*OT)[TCP], const uint8_t (*IDXT)[TC],
                                                const uint8_t (*IDX)[IDXB])
{
    constexpr uint32_t DPB = ES;                          // dwords per column and block-row: four values
    constexpr uint32_t OTD = (TR / 8) * DPB;
    const uint32_t tid = threadIdx.x;
    const uint32_t cols_valid = min((uint32_t)TC, d.cols - col0);
    const uint32_t brs_valid = min((uint32_t)(TR / 8), (d.rows - row0) / 8);
    const uint32_t rows_valid = brs_valid * 8;
    {
        const size_t pitch_b = (size_t)(d.rows / 8) * 4 * ES;          // bytes per row of valsT
        char *dst = (char *)d.valsT + (size_t)col0 * pitch_b + (size_t)(row0 / 8) * 4 * ES;
        if (brs_valid == TR / 8 && (pitch_b & 15) == 0 && (((uintptr_t)dst) & 15) == 0) {
            constexpr uint32_t CH = OTD / 4;                           // 16-byte pieces per column
            for (uint32_t j = tid; j < cols_valid * CH; j += NT) {
                const uint32_t cc = j / CH, part = j % CH;
                const u32x4 v = {OT[4 * part][cc], OT[4 * part + 1][cc], OT[4 * part + 2][cc], OT[4 * part + 3][cc]};
                stream_store(v, (u32x4 *)(dst + (size_t)cc * pitch_b + 16 * part));
            }
        } else {
            const uint32_t rd = brs_valid * DPB;                       // dwords per column
            for (uint32_t j = tid; j < cols_valid * rd; j += NT) {
                const uint32_t cc = j / rd, x = j - cc * rd;
                *(uint32_t *)(dst + (size_t)cc * pitch_b + 4 * x) = OT[x][cc];
            }
        }
    }
    {
        const size_t pitch = ((size_t)(d.cols / 8) * 12 + 7) / 8;
        const uint32_t nb = ((cols_valid / 8) * 12 + 7) / 8;
        unsigned char *dst = (unsigned char *)d.idx + (size_t)row0 * pitch + (size_t)(col0 / 8) * 12 / 8;
        if ((nb & 3) == 0 && (pitch & 3) == 0 && (((uintptr_t)dst) & 3) == 0) {
            const uint32_t nd = nb / 4;
            for (uint32_t j = tid; j < rows_valid * nd; j += NT) {
                const uint32_t r = j / nd, x = j - r * nd;
                *(uint32_t *)(dst + (size_t)r * pitch + 4 * x) = ((const uint32_t *)&IDX[r][0])[x];
            }
        } else {
            for (uint32_t j = tid; j < rows_valid * nb; j += NT) {
                const uint32_t r = j / nb, x = j - r * nb;
                dst[(size_t)r * pitch + x] = IDX[r][x];
            }
        }
    }
    {
        constexpr uint32_t PB = (IDXTB % 8 == 0) ? 8 : 4;              // bytes per store
        static_assert(IDXTB % PB == 0, "a tile column's position bytes are whole pieces");
        const size_t pitch = ((size_t)(d.rows / 8) * 12 + 7) / 8;
        const uint32_t nb = (brs_valid * 12 + 7) / 8;
        unsigned char *dst = (unsigned char *)d.idxT + (size_t)col0 * pitch + (size_t)(row0 / 8) * 12 / 8;
        if (nb == IDXTB && (pitch & (PB - 1)) == 0 && (((uintptr_t)dst) & (PB - 1)) == 0) {
            for (uint32_t j = tid; j < cols_valid * (IDXTB / PB); j += NT) {
                const uint32_t piece = j / cols_valid, cc = j - piece * cols_valid;
                uint32_t v[PB / 4];
#pragma unroll
                for (uint32_t h = 0; h < PB / 4; h++) {
                    v[h] = 0;
#pragma unroll
                    for (uint32_t k = 0; k < 4; k++)
                        v[h] |= (uint32_t)IDXT[PB * piece + 4 * h + k][cc] << (8 * k);
                }
                if constexpr (PB == 8) {
                    u32x2 vv;
                    vv.x = v[0];
                    vv.y = v[1];
                    *(u32x2 *)(dst + (size_t)cc * pitch + 8 * piece) = vv;
                } else {
                    *(uint32_t *)(dst + (size_t)cc * pitch + 4 * piece) = v[0];
                }
            }
        } else {
            for (uint32_t j = tid; j < cols_valid * nb; j += NT) {
                const uint32_t x = j / cols_valid, cc = j - x * cols_valid;
                dst[(size_t)cc * pitch + x] = IDXT[x][cc];
            }
        }
    }
}

// APPROX = false: tmask_apply_pack (ARGS = PackArgs, the mask is read).  APPROX = true: tmask_approx_pack
// (ARGS = FusedArgs): the keep flags come from Algorithm 1 in its threshold form (approx_half_bf16) on the
// lane's block; the mask is written if WMASK, the kept magnitudes' sum goes to the workgroup's partial.
template <int FMT, bool APPROX, bool WMASK, typename ARGS>
__global__ __launch_bounds__(kThreads) void pack48_bf16_kernel(const ARGS args)
{
    using PG = Pack8Geo;
    constexpr int ES = 2, S = PG::S, LPR = PG::LPR, NSTEP = PG::NSTEP, TR = PG::TR, TC = PG::TC, OTD = PG::OTD,
                  TCP = PG::TCP, IDXB = PG::IDXB, IDXTB = PG::IDXTB;

    __shared__ __attribute__((aligned(16))) uint32_t OT[OTD][TCP];      // [position down the column][column]
    __shared__ __attribute__((aligned(16))) uint8_t IDXT[IDXTB][TC];    // [byte of the column's bit string][column]
    __shared__ __attribute__((aligned(16))) uint8_t IDX[TR][IDXB];
    __shared__ __attribute__((aligned(16))) u32x4 LUTS[256];
    __shared__ uint16_t LUTC[256];
    __shared__ double red[kThreads / 64];

    const uint32_t tid = threadIdx.x, l = tid & 63u;
    // ---- the table: entry m describes the slots for the set m of kept positions (the kept ones in order, at most
    //      four; if fewer, the lowest-numbered other positions as fillers: choose_slots, worked out once per entry) ----
    {
        uint32_t sel, chosen;
        choose_slots<8>(tid, 4u, sel, chosen);
        uint32_t sa0 = 0x0C0C0C0Cu, sa1 = 0x0C0C0C0Cu, sb0 = 0x0C0C0C0Cu, sb1 = 0x0C0C0C0Cu, code = 0, s = 0;
#pragma unroll
        for (uint32_t p = 0; p < 8; p++) {
            if (((chosen >> p) & 1u) && s < 4u) {
                const uint32_t b = 2u * (p & 3u);
                const uint32_t pair = (b | ((b + 1u) << 8)) << (16u * (s & 1u));
                const uint32_t clear = ~(0xFFFFu << (16u * (s & 1u)));
                if (p < 4) {          // first half of the group: dwords 0 and 1
                    if (s < 2u) sa0 = (sa0 & clear) | pair; else sa1 = (sa1 & clear) | pair;
                } else {
                    if (s < 2u) sb0 = (sb0 & clear) | pair; else sb1 = (sb1 & clear) | pair;
                }
                code |= p << (3u * s);
                s++;
            }
        }
        LUTS[tid] = u32x4{sa0, sb0, sa1, sb1};
        LUTC[tid] = (uint16_t)code;
    }

    const uint32_t tile = blockIdx.x;
    const PackDev d = args.d[find_pack_desc(args, tile)];
    const uint32_t tl = tile - d.tile0;
    uint32_t ty, tx;
    tile_coords<APPROX ? 1 : 2>(tl, d.tiles_x, (d.rows + TR - 1) / TR, kPackRunRows / TR, ty, tx);
    const uint32_t row0 = ty * TR, col0 = tx * TC;
    const uint32_t w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t strip = l % (uint32_t)S, sub = l / (uint32_t)S;
    const uint32_t q2 = w * LPR + sub;                   // this lane's run of NSTEP block-rows inside the tile
    const uint32_t tcol = strip * 8u;
    const uint32_t col = col0 + tcol;
    const bool strip_ok = col < d.cols;
    const size_t pitchW = (size_t)(d.cols / 8) * 4;      // elements per row of vals
    const size_t lane_w = (size_t)sub * (8u * NSTEP) * d.ld * ES + strip * 16u;
    const size_t lane_m = (size_t)sub * (8u * NSTEP) * d.mask_ld + (FMT == kMaskU8 ? tcol : (col >> 3));
    const size_t lane_v = (size_t)sub * (8u * NSTEP) * pitchW * ES + strip * 8u;
    const size_t mcol0 = FMT == kMaskU8 ? col0 : 0;
    __syncthreads();                                      // the table is complete

    // ---- loads: both blocks of the lane first; when the mask is computed here, the second block's rows are
    // requested only after the first block's thresholds are done (they would occupy registers meanwhile) ----
    u32x4 raw[NSTEP][8];
    uint32_t mk0[NSTEP][8], mk1[NSTEP][8];               // U8: the row's eight mask bytes; BITS: the byte in mk0
    bool okq[NSTEP];
    auto issue = [&](int q) {
        const uint32_t wrow = row0 + 8u * NSTEP * LPR * w + 8u * (uint32_t)q;     // scalar: the row of sub-run 0
        const uint32_t row = wrow + 8u * NSTEP * sub;
        okq[q] = strip_ok && row < d.rows;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            raw[q][i] = u32x4{0u, 0u, 0u, 0u};
            mk0[q][i] = mk1[q][i] = 0;
        }
        if (okq[q]) {
#pragma unroll
            for (int i = 0; i < 8; i++) {
                raw[q][i] = __builtin_nontemporal_load(
                    (const u32x4 *)((const char *)d.w + ((size_t)(wrow + i) * d.ld + col0) * ES + lane_w));
                if constexpr (APPROX)
                    continue;
                const unsigned char *mp = (const unsigned char *)d.mask + (size_t)(wrow + i) * d.mask_ld + mcol0 + lane_m;
                if constexpr (FMT == kMaskU8) {
                    const u32x2 mv = __builtin_nontemporal_load((const u32x2 *)mp);
                    mk0[q][i] = mv.x;
                    mk1[q][i] = mv.y;
                } else {
                    mk0[q][i] = (uint32_t)*mp;
                }
            }
        }
    };
    issue(0);
    if constexpr (!APPROX)
        issue(1);
    static_assert(NSTEP == 2, "the load schedule above is written for two blocks per lane");

    float acc = 0.f;
    uint32_t tcode[8];                                    // position bits of the lane's columns, 12 per block-row
#pragma unroll
    for (int c = 0; c < 8; c++)
        tcode[c] = 0;

#pragma unroll
    for (int q = 0; q < NSTEP; q++) {
        const uint32_t brl = NSTEP * q2 + (uint32_t)q;   // block-row inside the tile
        const uint32_t wrow = row0 + 8u * NSTEP * LPR * w + 8u * (uint32_t)q;
        const bool ok = okq[q];
        if constexpr (APPROX) {
            // Algorithm 1 on the lane's block: 0/1 bytes per row, stored as the mask on request.  (Lanes outside
            // the matrix hold zeros: their flags are discarded below and their sum is zero.)
            acc += approx_half_bf16<8>(raw[q], 0u, [&](int i, uint32_t b0, uint32_t b1) {
                mk0[q][i] = b0;
                mk1[q][i] = b1;
                // the flags exist as bytes from here on (otherwise the compiler carries the compare results of all
                // 64 entries as lane masks into the compaction below and runs out of scalar registers)
                asm volatile("" : "+v"(mk0[q][i]), "+v"(mk1[q][i]));
                if constexpr (WMASK) {
                    if (ok) {
                        unsigned char *mp = (unsigned char *)const_cast<void *>(d.mask) + (size_t)(wrow + i) * d.mask_ld + mcol0 + lane_m;
                        if constexpr (FMT == kMaskU8) {
                            u32x2 v;
                            v.x = b0;
                            v.y = b1;
                            stream_store(v, (u32x2 *)mp);
                        } else {
                            *mp = (unsigned char)(bytes4_to_bits(b0) | (bytes4_to_bits(b1) << 4));
                        }
                    }
                }
            });
            // the sum is needed only at the very end, and only if an objective is asked for: left alone, the compiler
            // moves all its additions there and keeps every keep flag and magnitude alive until then
            asm volatile("" : "+v"(acc));
            __builtin_amdgcn_sched_barrier(0);
            if (q == 0)
                issue(1);
            __builtin_amdgcn_sched_barrier(0);
        }
        // keep bits per row, and the block with its pruned values zeroed
        uint32_t rb[8], e[8][4];
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const uint32_t dw[4] = {raw[q][i].x, raw[q][i].y, raw[q][i].z, raw[q][i].w};
            if constexpr (FMT == kMaskU8 || APPROX) {
                // bytes -> 0x00 / 0xFF, then every byte doubled into a halfword mask
                uint32_t f[2] = {mk0[q][i], mk1[q][i]};
#pragma unroll
                for (int h = 0; h < 2; h++) {
                    uint32_t nz = (((f[h] & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | f[h]) & 0x80808080u;
                    f[h] = nz | (nz - (nz >> 7));
                }
                rb[i] = bytes4_to_bits(f[0]) | (bytes4_to_bits(f[1]) << 4);
                e[i][0] = dw[0] & __builtin_amdgcn_perm(0u, f[0], 0x01010000u);
                e[i][1] = dw[1] & __builtin_amdgcn_perm(0u, f[0], 0x03030202u);
                e[i][2] = dw[2] & __builtin_amdgcn_perm(0u, f[1], 0x01010000u);
                e[i][3] = dw[3] & __builtin_amdgcn_perm(0u, f[1], 0x03030202u);
            } else {
                rb[i] = mk0[q][i];
#pragma unroll
                for (int h = 0; h < 4; h++) {
                    const uint32_t t = rb[i] >> (2 * h);
                    e[i][h] = dw[h] & (((0u - (t & 1u)) & 0xFFFFu) | ((0u - ((t >> 1) & 1u)) << 16));
                }
            }
        }
        // ---- W: the rows ----
#pragma unroll
        for (int i = 0; i < 8; i++) {
            uint32_t o0, o1, code;
            compact_4of8(rb[i], e[i][0], e[i][1], e[i][2], e[i][3], LUTS, LUTC, o0, o1, code);
            if (!ok)
                code = 0;                                 // nothing of this strip may show up in a row's padding bits
            const uint32_t other = quad_xor<1>(code);
            if (ok) {
                u32x2 v;
                v.x = o0;
                v.y = o1;
                stream_store(v, (u32x2 *)((char *)d.vals + ((size_t)(wrow + i) * pitchW + (size_t)(col0 / 8) * 4) * ES + lane_v));
            }
            // two lanes share three bytes: the even one writes the first two, the odd one the third
            uint8_t *ip = &IDX[8 * brl + i][3 * (strip >> 1)];
            if ((l & 1u) == 0) {
                ip[0] = (uint8_t)code;
                ip[1] = (uint8_t)((code >> 8) | (other << 4));
            } else {
                ip[2] = (uint8_t)(code >> 4);
            }
        }
        // ---- W^T: the columns ----
        uint32_t cx, cy;
        transpose_bits8(rb, cx, cy);
        uint32_t oc0[8], oc1[8];
#pragma unroll
        for (int c = 0; c < 8; c++) {
            const uint32_t kb = ((c < 4 ? cx : cy) >> (8 * (c & 3))) & 0xFFu;
            const uint32_t selh = (c & 1) ? 0x07060302u : 0x05040100u;     // the column's halfword of two rows
            const uint32_t d0 = __builtin_amdgcn_perm(e[1][c >> 1], e[0][c >> 1], selh);
            const uint32_t d1 = __builtin_amdgcn_perm(e[3][c >> 1], e[2][c >> 1], selh);
            const uint32_t d2 = __builtin_amdgcn_perm(e[5][c >> 1], e[4][c >> 1], selh);
            const uint32_t d3 = __builtin_amdgcn_perm(e[7][c >> 1], e[6][c >> 1], selh);
            uint32_t code;
            compact_4of8(kb, d0, d1, d2, d3, LUTS, LUTC, oc0[c], oc1[c], code);
            tcode[c] |= (ok ? code : 0u) << (12 * q);
        }
        *(u32x4 *)&OT[2 * brl][tcol] = u32x4{oc0[0], oc0[1], oc0[2], oc0[3]};
        *(u32x4 *)&OT[2 * brl][tcol + 4] = u32x4{oc0[4], oc0[5], oc0[6], oc0[7]};
        *(u32x4 *)&OT[2 * brl + 1][tcol] = u32x4{oc1[0], oc1[1], oc1[2], oc1[3]};
        *(u32x4 *)&OT[2 * brl + 1][tcol + 4] = u32x4{oc1[4], oc1[5], oc1[6], oc1[7]};
    }
    // the lane's two block-rows are neighbours: 24 position bits = three whole bytes per column
#pragma unroll
    for (int t = 0; t < 3; t++) {
        u32x2 v;
        v.x = ((tcode[0] >> (8 * t)) & 0xFFu) | (((tcode[1] >> (8 * t)) & 0xFFu) << 8) |
              (((tcode[2] >> (8 * t)) & 0xFFu) << 16) | (((tcode[3] >> (8 * t)) & 0xFFu) << 24);
        v.y = ((tcode[4] >> (8 * t)) & 0xFFu) | (((tcode[5] >> (8 * t)) & 0xFFu) << 8) |
              (((tcode[6] >> (8 * t)) & 0xFFu) << 16) | (((tcode[7] >> (8 * t)) & 0xFFu) << 24);
        *(u32x2 *)&IDXT[3 * q2 + t][tcol] = v;
    }
    __syncthreads();

    pack48_copy_out<ES, TR, TC, TCP, IDXB, IDXTB, kThreads>(d, row0, col0, OT, IDXT, IDX);
    if constexpr (APPROX) {
        if (args.partials) {
            const double t = block_sum_f32(acc, red);
            if (threadIdx.x == 0)
                ((double *)args.partials)[args.partial0 + tile] = t;
        }
    }
}


// =================================================================================================
// fp32, M = 8, N = 4.  A strip of 16 bytes is half a group, so two neighbouring lanes hold an 8 x 8 block
// per step (8 rows x 4 columns each).
//   W^T : a lane owns four whole column groups.  The group's set of kept rows indexes a 256-entry table of
//         position codes (the rule "kept in order, at most four, then the lowest unused positions" is
//         worked out once per entry when the workgroup builds the table); slot s sits at most four rows
//         below row s, so a five-way select picks it.
//   W   : a row group spans the two lanes.  They exchange their keep nibbles (all eight rows in one
//         dword) and the two values the other may need: the even lane writes slots 0 and 1, which come
//         from positions 0..5, the odd lane slots 2 and 3, from positions 2..7.  Each lane stores 8 bytes
//         per row, so a wavefront's stores are contiguous as in the other pack kernels.
// Staging and copy-out as in pack48_bf16_kernel.
// =================================================================================================
constexpr int kPack8F32Strips = 64;   // tile width in strips (32: 123 against 121 us on 8192 x 8192)

template <int S, int QN = 2, int NW = 4>
struct Pack8F32Geo {
    static constexpr int LPR = 64 / S;                 // runs of block-rows a wavefront covers at a time
    static constexpr int NT = 64 * NW;
    static constexpr int TR = 8 * QN * LPR * NW, TC = S * 4;
    static constexpr int NBR = TR / 8;                 // block-rows per tile
    static constexpr int OTD = NBR * 4;                // dwords per column of W^T in the tile
    static constexpr int TCP = TC + 4;
    static constexpr int IDXB = (S / 2) * 12 / 8;      // position bytes per tile row (S / 2 groups)
    static constexpr int IDXTB = NBR * 12 / 8;         // position bytes per tile column
};

// All-ones if bit `pos` of x is set, else zero (one v_bfe_i32), and m ? a : b bit by bit (one v_bfi_b32, written as an
// instruction so that the compiler does not turn chains of such selects into indexed loads from a copy in scratch).
__device__ __forceinline__ uint32_t bit_mask(uint32_t x, uint32_t pos) { return (uint32_t)__builtin_amdgcn_sbfe((int)x, pos, 1u); }
__device__ __forceinline__ uint32_t bit_select(uint32_t m, uint32_t a, uint32_t b)
{
    uint32_t r;
    asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(r) : "v"(m), "v"(a), "v"(b));
    return r;
}

// bits 0, 4, ..., 28 of y gathered into bits 0..7
__device__ __forceinline__ uint32_t gather_every_fourth_bit(uint32_t y)
{
    y &= 0x11111111u;
    y = (y | (y >> 3)) & 0x03030303u;
    y = (y | (y >> 6)) & 0x000F000Fu;
    return (y | (y >> 12)) & 0xFFu;
}

// APPROX = false: tmask_apply_pack (ARGS = PackArgs, the mask is read).  APPROX = true: tmask_approx_pack (ARGS =
// FusedArgs): the keep flags come from Algorithm 1 in its threshold form on the lane pair's block
// (approx_half_f32; a wavefront in which some line has a tie across its cut redoes its blocks with approx_half_f32_ties),
// the mask is written if WMASK, the kept magnitudes' sum goes to the workgroup's partial.
template <int FMT, int S, bool APPROX, bool WMASK, typename ARGS>
__global__ __launch_bounds__(256) void pack48_f32_kernel(const ARGS args)
{
    using PG = Pack8F32Geo<S>;
    constexpr int ES = 4, QN = 2, LPR = PG::LPR, TR = PG::TR, TC = PG::TC, OTD = PG::OTD, TCP = PG::TCP,
                  IDXB = PG::IDXB, IDXTB = PG::IDXTB, NT = PG::NT;
    static_assert(NT == 256 && S % 4 == 0, "the table has one entry per thread; two groups share a quad");

    __shared__ __attribute__((aligned(16))) uint32_t OT[OTD][TCP];      // [position down the column][column]
    __shared__ __attribute__((aligned(16))) uint8_t IDXT[IDXTB][TC];    // [byte of the column's bit string][column]
    __shared__ __attribute__((aligned(16))) uint8_t IDX[TR][IDXB];
    __shared__ uint16_t LUT[256];
    __shared__ double red[NT / 64];

    const uint32_t tid = threadIdx.x, l = tid & 63u;
    // ---- the table: entry m = position codes (3 bits per slot) of the four slots for the set m of kept positions ----
    {
        uint32_t chosen = 0, cnt = 0;
#pragma unroll
        for (uint32_t p = 0; p < 8; p++)
            if (((tid >> p) & 1u) && cnt < 4u) {
                chosen |= 1u << p;
                cnt++;
            }
#pragma unroll
        for (uint32_t p = 0; p < 8; p++)
            if (!((tid >> p) & 1u) && cnt < 4u) {
                chosen |= 1u << p;
                cnt++;
            }
        uint32_t code = 0, sl = 0;
#pragma unroll
        for (uint32_t p = 0; p < 8; p++)
            if ((chosen >> p) & 1u) {
                code |= p << (3u * sl);
                sl++;
            }
        LUT[tid] = (uint16_t)code;
    }

    const uint32_t tile = blockIdx.x;
    const PackDev d = args.d[find_pack_desc(args, tile)];
    const uint32_t tl = tile - d.tile0;
    uint32_t ty, tx;
    tile_coords(tl, d.tiles_x, (d.rows + TR - 1) / TR, kPackRunRows / TR, ty, tx);
    const uint32_t row0 = ty * TR, col0 = tx * TC;
    const uint32_t w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t strip = l % (uint32_t)S, sub = l / (uint32_t)S;
    const uint32_t q2 = w * LPR + sub;                   // this lane's run of QN block-rows inside the tile
    const uint32_t tcol = strip * 4u;
    const uint32_t col = col0 + tcol;
    const bool strip_ok = col < d.cols;
    const bool odd = (l & 1u) != 0;                      // second half of the row groups
    const lanemask_t odd_m = 0xAAAAAAAAAAAAAAAAull;
    const uint32_t sel_xor = odd ? 0x900u : 0u, sel_shift = odd ? 6u : 0u;
    const size_t pitchW = (size_t)(d.cols / 8) * 4;      // elements per row of vals
    const size_t lane_w = (size_t)sub * (8u * QN) * d.ld * ES + strip * 16u;
    const size_t lane_m = (size_t)sub * (8u * QN) * d.mask_ld + (FMT == kMaskU8 ? tcol : (col >> 3));
    const size_t lane_v = (size_t)sub * (8u * QN) * pitchW * ES + strip * 8u;
    const size_t mcol0 = FMT == kMaskU8 ? col0 : 0;
    __syncthreads();                                      // the table is complete

    u32x4 raw[QN][8];
    uint32_t mk[QN][8];                                   // U8: the row's four mask bytes; BITS: the lane's nibble
    bool okq[QN];
#pragma unroll
    for (int q = 0; q < QN; q++) {
        const uint32_t wrow = row0 + 8u * QN * LPR * w + 8u * (uint32_t)q;     // scalar: the row of sub-run 0
        const uint32_t row = wrow + 8u * QN * sub;
        okq[q] = strip_ok && row < d.rows;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            raw[q][i] = u32x4{0u, 0u, 0u, 0u};
            mk[q][i] = 0;
        }
        if (okq[q]) {
#pragma unroll
            for (int i = 0; i < 8; i++) {
                raw[q][i] = __builtin_nontemporal_load(
                    (const u32x4 *)((const char *)d.w + ((size_t)(wrow + i) * d.ld + col0) * ES + lane_w));
                if constexpr (APPROX)
                    continue;
                const unsigned char *mp = (const unsigned char *)d.mask + (size_t)(wrow + i) * d.mask_ld + mcol0 + lane_m;
                if constexpr (FMT == kMaskU8)
                    mk[q][i] = __builtin_nontemporal_load((const uint32_t *)mp);
                else
                    mk[q][i] = ((uint32_t)*mp >> (col & 4u)) & 0xFu;
            }
        }
    }
    float acc = 0.f;

    uint32_t tcode[4] = {0u, 0u, 0u, 0u};                 // position bits of the lane's columns, 12 per block-row
#pragma unroll
    for (int q = 0; q < QN; q++) {
        const uint32_t brl = QN * q2 + (uint32_t)q;      // block-row inside the tile
        const uint32_t wrow = row0 + 8u * QN * LPR * w + 8u * (uint32_t)q;
        const bool ok = okq[q];
        if constexpr (APPROX) {
            // Algorithm 1 on the lane pair's block (lanes outside the matrix hold zeros: their flags are discarded
            // below and their sum is zero)
            uint32_t a[8][4];
#pragma unroll
            for (int i = 0; i < 8; i++) {
                a[i][0] = raw[q][i].x & 0x7FFFFFFFu;
                a[i][1] = raw[q][i].y & 0x7FFFFFFFu;
                a[i][2] = raw[q][i].z & 0x7FFFFFFFu;
                a[i][3] = raw[q][i].w & 0x7FFFFFFFu;
            }
            float part = 0.f;
            const bool tie = approx_half_f32<8>(a, l & 1u, mk[q], part);
            if (__any(tie))
                approx_half_f32_ties<8>(a, l & 1u, mk[q], part);
            acc += part;
            // the flags exist as bytes from here on, and the sum is complete (see pack48_bf16_kernel)
#pragma unroll
            for (int i = 0; i < 8; i++)
                asm volatile("" : "+v"(mk[q][i]));
            asm volatile("" : "+v"(acc));
            if constexpr (WMASK) {
                if (ok) {
#pragma unroll
                    for (int i = 0; i < 8; i++) {
                        unsigned char *mp = (unsigned char *)const_cast<void *>(d.mask) + (size_t)(wrow + i) * d.mask_ld + mcol0 + lane_m;
                        if constexpr (FMT == kMaskU8) {
                            stream_store(mk[q][i], (uint32_t *)mp);
                        } else {
                            const uint32_t nb = bytes4_to_bits(mk[q][i]);
                            const uint32_t ob = quad_xor<1>(nb);
                            if (!odd)
                                *mp = (unsigned char)(nb | (ob << 4));
                        }
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // keep nibbles of the eight rows in one dword, and the block with its pruned values zeroed
        uint32_t e[8][4], nib32 = 0;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const uint32_t dw[4] = {raw[q][i].x, raw[q][i].y, raw[q][i].z, raw[q][i].w};
            uint32_t nib;
            if constexpr (FMT == kMaskU8 || APPROX)
                nib = bytes4_to_bits(mk[q][i]);
            else
                nib = mk[q][i];
#pragma unroll
            for (int c = 0; c < 4; c++)
                e[i][c] = dw[c] & (0u - ((nib >> c) & 1u));
            nib32 |= nib << (4 * i);
        }
        const uint32_t other32 = quad_xor<1>(nib32);
        const uint32_t lo32 = odd ? other32 : nib32, hi32 = odd ? nib32 : other32;
        // ---- W: the rows ----
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const uint32_t kb = ((lo32 >> (4 * i)) & 0xFu) | (((hi32 >> (4 * i)) & 0xFu) << 4);
            uint32_t code = LUT[kb];
            // what the other lane may need of this one: positions 2, 3 from the even lane, 4, 5 from the odd one
            const uint32_t r0 = quad_xor<1>(lm_select(odd_m, e[i][0], e[i][2]));
            const uint32_t r1 = quad_xor<1>(lm_select(odd_m, e[i][1], e[i][3]));
            // selector = position (even lane: 0..5, 4 and 5 are the received values) or position ^ 4 (odd lane:
            // 4..7 -> own 0..3, 2 and 3 -> 6 and 7, the received values)
            const uint32_t x = (code ^ sel_xor) >> sel_shift;
            uint32_t o[2];
#pragma unroll
            for (int t = 0; t < 2; t++) {
                // (selects written as instructions: as plain conditionals the compiler turns them into indexed
                // loads from a copy of the block in scratch memory)
                const uint32_t b0 = bit_mask(x, 3 * t), b1 = bit_mask(x, 3 * t + 1), b2 = bit_mask(x, 3 * t + 2);
                const uint32_t t0 = bit_select(b0, e[i][1], e[i][0]);
                const uint32_t t1 = bit_select(b0, e[i][3], e[i][2]);
                const uint32_t t2 = bit_select(b0, r1, r0);
                const uint32_t u = bit_select(b1, t1, t0);
                o[t] = bit_select(b2, t2, u);
            }
            if (!ok)
                code = 0;                                 // nothing of this strip may show up in a row's padding bits
            const uint32_t other = quad_xor<2>(code);     // the code of the quad's other group
            if (ok) {
                u32x2 v;
                v.x = o[0];
                v.y = o[1];
                stream_store(v, (u32x2 *)((char *)d.vals + ((size_t)(wrow + i) * pitchW + (size_t)(col0 / 8) * 4) * ES + lane_v));
            }
            // the two groups of a quad share three bytes: lane 0 writes the first two, lane 2 the third
            uint8_t *ip = &IDX[8 * brl + i][3 * (strip >> 2)];
            if ((l & 3u) == 0) {
                ip[0] = (uint8_t)code;
                ip[1] = (uint8_t)((code >> 8) | (other << 4));
            } else if ((l & 3u) == 2u) {
                ip[2] = (uint8_t)(code >> 4);
            }
        }
        // ---- W^T: the columns ----
        uint32_t oc[4][4];
#pragma unroll
        for (int c = 0; c < 4; c++) {
            const uint32_t kb = gather_every_fourth_bit(nib32 >> c);
            const uint32_t code = LUT[kb];
            const uint32_t gaps = code - 0x688u;          // slot s sits (position - s) rows below row s: 0..4 each
#pragma unroll
            for (int sl = 0; sl < 4; sl++) {
                const uint32_t b0 = bit_mask(gaps, 3 * sl), b1 = bit_mask(gaps, 3 * sl + 1), b2 = bit_mask(gaps, 3 * sl + 2);
                const uint32_t t0 = bit_select(b0, e[sl + 1][c], e[sl][c]);
                const uint32_t t1 = bit_select(b0, e[sl + 3][c], e[sl + 2][c]);
                const uint32_t u = bit_select(b1, t1, t0);
                oc[sl][c] = bit_select(b2, e[sl + 4][c], u);
            }
            tcode[c] |= (ok ? code : 0u) << (12 * q);
        }
#pragma unroll
        for (int sl = 0; sl < 4; sl++)
            *(u32x4 *)&OT[4 * brl + sl][tcol] = u32x4{oc[sl][0], oc[sl][1], oc[sl][2], oc[sl][3]};
    }
    // the lane's two block-rows are neighbours: 24 position bits = three whole bytes per column
    static_assert(QN == 2, "three bytes per column and lane");
#pragma unroll
    for (int t = 0; t < 3; t++)
        *(uint32_t *)&IDXT[3 * q2 + t][tcol] = ((tcode[0] >> (8 * t)) & 0xFFu) | (((tcode[1] >> (8 * t)) & 0xFFu) << 8) |
                                               (((tcode[2] >> (8 * t)) & 0xFFu) << 16) | (((tcode[3] >> (8 * t)) & 0xFFu) << 24);
    __syncthreads();
    pack48_copy_out<ES, TR, TC, TCP, IDXB, IDXTB, NT>(d, row0, col0, OT, IDXT, IDX);
    if constexpr (APPROX) {
        if (args.partials) {
            const double t = block_sum_f32(acc, red);
            if (threadIdx.x == 0)
                ((double *)args.partials)[args.partial0 + tile] = t;
        }
    }
}

}  // namespace tmask

// tmask_apply_pack: W (.) S and compression of W and W^T into N values + N positions per group of M.
//
// The paper (arXiv 2102.08124, Sec. 1 (Eq. 1) and Sec. 4) only states why both operands are needed: the
// forward product reads W and the backward product reads W^T, and a transposable mask leaves N
// non-zeros in every M contiguous elements of both.  The storage format is this library's own and
// is described in include/tmask.h.
//
// One workgroup packs a 64-row x 256-byte tile (64 fp32 or 128 bf16 columns):
//   A  coalesced 16-byte loads of W and of the mask; masked values and 0/1 flags go to LDS
//   C  every thread pulls its row-direction units (one row x one group of M columns) and its
//      column-direction units (one group of M rows x one column) from LDS into registers
//   E  each unit is compacted (kept entries, then lowest unused positions as +0 fillers, in position
//      order) and scattered into LDS staging: values row-major for W, column-major for W^T, index
//      bits OR-ed into per-row bit strings
//   G  staging is streamed out with coalesced stores (runs of 128..256 bytes per output row)
#pragma once
#include "tmask_device.hpp"

namespace tmask {

constexpr int kMaxPackBatch = 224;  // descriptors of 72 bytes, passed by value as kernel argument (16 KiB)
constexpr int kPackTR = 64;

struct PackDev {
    const void *w;
    const void *mask;
    void *vals, *idx, *valsT, *idxT;
    uint32_t rows, cols, ld, mask_ld;
    uint32_t tiles_x;   // tiles per tile-row
    uint32_t tile0;     // first workgroup of this matrix inside the launch
};

struct PackArgs {
    PackDev d[kMaxPackBatch];
    CoarseIndex ci;
    uint32_t n;
    uint32_t N;
};
static_assert(sizeof(PackArgs) <= 16384 + 2048, "descriptor table is sized to stay a small kernel argument");

// Arguments of the kernels that compute the mask themselves (tmask_approx_pack).
struct FusedArgs {
    PackDev d[kMaxPackBatch];   // mask = output here (may be null when WMASK is false)
    CoarseIndex ci;
    uint32_t n;
    uint32_t partial0;          // index of this launch's first partial in the workspace
    void *partials;             // one double per workgroup, or null
};
static_assert(sizeof(FusedArgs) <= 16384 + 2048, "descriptor table is sized to stay a small kernel argument");


// Tile number inside a matrix -> tile coordinates, for the kernels that write W^T in short runs per column.
// Workgroups go to the eight XCDs round-robin, so tile numbers t, t + 8, t + 16, ... run on one XCD one after
// the other.  They walk down a column band of tiles in runs of `run` tiles (4096 rows), band x, 8 + x, ... for
// XCD x, then the next 4096 rows: the pieces that the tiles of a run write into one row of W^T are neighbours
// in memory and arrive close in time, which the memory system rewards (fp32 2:4 pack: 66 -> 73 % of the HBM
// peak at 8192 x 8192; shorter runs lose it again, full-height runs cost the bf16 kernels 5 points).
// Bands beyond the last multiple of eight are walked column by column.
// ADJ > 1: an XCD takes ADJ neighbouring tile columns together, one after the other at each height: for kernels whose
// tiles are narrower than a cache line of the mask or of an index row, so that the tiles sharing such a line meet in
// one L2 instead of each fetching (or partly writing) it.  The generic kernel (256-byte tiles: 64 mask bytes and 16
// index bytes per tile row at fp32 8:16) fetched 1.20x and wrote 1.14x its algorithmic bytes without it; with four
// columns together 8192^2 fp32 8:16 goes from 145 to 121 us, 16384^2 from 715 to 505 us, 3:8 from 192 to 143 us.  The
// kernels with 1 KB tiles lose with it (fp32 2:4: 107 -> 115 us), except the bf16 4:8 pack with two (78 -> 73 us).
constexpr uint32_t kPackRunRows = 4096;


// Which descriptor does workgroup `tile` belong to (PackArgs or FusedArgs): coarse index, then a short binary search.
template <typename Args>
__device__ __forceinline__ int find_pack_desc(const Args &args, uint32_t tile)
{
    const uint32_t e = args.ci.e[tile >> args.ci.shift];
    int lo = (int)(e & 0xFFFFu), hi = (int)(e >> 16);
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (args.d[mid].tile0 <= tile)
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo;
}

template <uint32_t ADJ = 1>
__device__ __forceinline__ void tile_coords(uint32_t tl, uint32_t tiles_x, uint32_t tiles_y, uint32_t run, uint32_t &ty,
                                            uint32_t &tx)
{
    const uint32_t bands8 = tiles_x / (8u * ADJ), full = bands8 * 8u * ADJ * tiles_y;
    if (tl < full) {
        const uint32_t x = tl & 7u, ka = tl >> 3;
        const uint32_t a = ka % ADJ, k = ka / ADJ;
        const uint32_t per_chunk = run * bands8;
        const uint32_t chunk = k / per_chunk, rk = k - chunk * per_chunk;
        const uint32_t rows_here = min(run, tiles_y - chunk * run);       // the last chunk may be shorter
        const uint32_t band = rk / rows_here;
        ty = chunk * run + (rk - band * rows_here);
        tx = (band * 8u + x) * ADJ + a;
    } else {
        const uint32_t r = tl - full;
        const uint32_t c = r / tiles_y;
        ty = r - c * tiles_y;
        tx = bands8 * 8u * ADJ + c;
    }
}

template <int M>
struct Log2 {
    static constexpr int v = (M == 4) ? 2 : (M == 8) ? 3 : (M == 16) ? 4 : 5;
};

// Which positions of a group of M fill its N slots.  kbits = keep flags (bit p = position p).
// sel    = kept positions that get a slot: all of them, or the first N if the mask (wrongly) keeps more;
// chosen = sel plus, if fewer than N are kept, the lowest-numbered other positions as +0 fillers.
template <int M>
__device__ __forceinline__ void choose_slots(uint32_t kbits, uint32_t N, uint32_t &sel, uint32_t &chosen)
{
    sel = kbits;
    uint32_t cnt = (uint32_t)__builtin_popcount(sel);
    while (cnt > N) {                                   // caller error, rare: drop the highest kept position
        sel &= ~(0x80000000u >> __builtin_clz(sel));
        cnt--;
    }
    uint32_t z = ~sel & (M == 32 ? 0xFFFFFFFFu : ((1u << (M & 31)) - 1u)), f = 0;
    for (uint32_t need = N - cnt; need > 0; need--) {   // approximate masks: usually zero to two rounds
        const uint32_t low = z & (0u - z);
        f |= low;
        z ^= low;
    }
    chosen = sel | f;
}

// ORs `nbits` (<= 60) bits of `code` into an LDS bit string at bit offset `off`.
__device__ __forceinline__ void lds_or_bits(uint32_t *words, uint32_t off, unsigned long long code)
{
    const uint32_t w = off >> 5, sh = off & 31u;
    const unsigned long long lo = code << sh;                       // bits landing in words w, w+1
    const uint32_t hi = sh ? (uint32_t)(code >> (64 - sh)) : 0u;    // bits landing in word w+2
    if ((uint32_t)lo)
        atomicOr(&words[w], (uint32_t)lo);
    if ((uint32_t)(lo >> 32))
        atomicOr(&words[w + 1], (uint32_t)(lo >> 32));
    if (hi)
        atomicOr(&words[w + 2], hi);
}

// NN = N when it is known at compile time (N = M/2: slot loops unrolled, a row group's values leave as 16-byte
// stores), 0 = any N (args.N).
// The BITS position bits of group number `g` of a line into the line's bit string (cleared beforehand): whole words are
// stored, anything else is ORed in.
template <int BITS>
__device__ __forceinline__ void put_code(uint32_t *words, uint32_t g, unsigned long long code)
{
    if constexpr (BITS % 32 == 0) {
#pragma unroll
        for (int w = 0; w < BITS / 32; w++)
            words[g * (BITS / 32) + w] = (uint32_t)(code >> (32 * w));
    } else {
        lds_or_bits(words, g * BITS, code);
    }
}

template <int DT, int M, int FMT, int NN = 0>
__global__ __launch_bounds__(kThreads) void pack_kernel(const PackArgs args)
{
    using T = typename std::conditional<DT == kF32, uint32_t, uint16_t>::type;
    constexpr int ES = sizeof(T);
    constexpr int C = 16 / ES;                 // elements per 16-byte chunk
    constexpr int TR = kPackTR;
    constexpr int TC = 256 / ES;               // tile columns
    constexpr int IB = Log2<M>::v;
    constexpr int GPT = TC / M;                // groups per tile row
    constexpr int BPT = TR / M;                // block-rows per tile
    constexpr int OTR = NN ? TR * NN / M : TR; // staged W^T values per column: N per block-row (at most M - 1 if N is not known)
    constexpr int OTP = OTR + 4 / ES;          // pitch of the transposed staging (bank-conflict free)
    constexpr int NMAX = NN ? NN : M - 1;      // slots per group the staging must hold
    constexpr int IDXW = (GPT * NMAX * IB + 31) / 32 + 2;
    constexpr int IDXTW = (BPT * NMAX * IB + 31) / 32 + 2 + 1;
    constexpr int NRU = (TR * GPT + kThreads - 1) / kThreads;   // row-direction units per thread
    constexpr int NCU = (BPT * TC + kThreads - 1) / kThreads;   // column-direction units per thread
    static_assert((TR * GPT % kThreads == 0 || TR * GPT < kThreads) && (BPT * TC % kThreads == 0 || BPT * TC < kThreads),
                  "units tile the workgroup, or there are fewer of them than threads (fp32 at M = 32)");
    // Position codes of a group: NN * IB bits.  Beyond 64 bits (16:32: 80) they are kept as two halves of NN / 2 slots,
    // which go into the bit string as groups number 2g and 2g + 1 of half the width.
    constexpr bool SPLIT = NN * IB > 64;
    constexpr int HS = SPLIT ? NN / 2 : NN;    // slots per code word
    static_assert(M < 32 || NN == 16, "M = 32 comes here at 16:32 only (whole bytes of position bits per tile row)");

    __shared__ __attribute__((aligned(16))) T V[TR][TC];   // masked tile
    __shared__ __attribute__((aligned(16))) uint8_t FN[TR][16];   // keep flags of each 16-byte chunk (C bits), 16 chunks per tile row
    __shared__ T OT[TC][OTP];
    __shared__ uint32_t IDX[TR][IDXW];
    __shared__ uint32_t IDXT[TC][IDXTW];

    // ---- which tile ----
    const uint32_t tile = blockIdx.x;
    const PackDev d = args.d[find_pack_desc(args, tile)];
    const uint32_t N = NN ? (uint32_t)NN : args.N;
    const uint32_t tl = tile - d.tile0;
    uint32_t ty, tx;
    tile_coords<4>(tl, d.tiles_x, (d.rows + TR - 1) / TR, kPackRunRows / TR, ty, tx);
    const uint32_t row0 = ty * TR, col0 = tx * TC;
    const uint32_t tid = threadIdx.x;
    const uint32_t g_valid = min((uint32_t)GPT, (d.cols - col0) / M);   // groups of this tile inside the matrix
    const uint32_t b_valid = min((uint32_t)BPT, (d.rows - row0) / M);
    const uint32_t r_valid = b_valid * M, c_valid = g_valid * M;

    // ---- A: load ----
    for (uint32_t k = tid; k < TR * IDXW; k += kThreads)
        (&IDX[0][0])[k] = 0;
    for (uint32_t k = tid; k < TC * IDXTW; k += kThreads)
        (&IDXT[0][0])[k] = 0;
    // all loads of the thread go out before the first is used, none inside a branch (its result would be waited for
    // at the join): chunks outside the matrix read chunk (0, 0) and are dropped
    constexpr int PASSES = TR / 16;
    u32x4 raws[PASSES];
    uint32_t mlo[PASSES], mhi[PASSES];
#pragma unroll
    for (int pass = 0; pass < PASSES; pass++) {
        const uint32_t r = pass * 16 + (tid >> 4), ch = tid & 15u;
        const uint32_t row = row0 + r, col = col0 + ch * C;
        const bool ok = row < d.rows && col < d.cols;
        const uint32_t rowc = ok ? row : 0u, colc = ok ? col : 0u;
        raws[pass] = __builtin_nontemporal_load((const u32x4 *)((const char *)d.w + ((size_t)rowc * d.ld + colc) * ES));
        mhi[pass] = 0;
        if constexpr (FMT == kMaskU8) {
            const char *mp = (const char *)d.mask + (size_t)rowc * d.mask_ld + colc;
            if constexpr (C == 4) {
                mlo[pass] = __builtin_nontemporal_load((const uint32_t *)mp);
            } else {
                const u32x2 mv = __builtin_nontemporal_load((const u32x2 *)mp);
                mlo[pass] = mv.x;
                mhi[pass] = mv.y;
            }
        } else {
            mlo[pass] = ((const unsigned char *)d.mask)[(size_t)rowc * d.mask_ld + (colc >> 3)];
        }
    }
#pragma unroll
    for (int pass = 0; pass < PASSES; pass++) {
        const uint32_t r = pass * 16 + (tid >> 4), ch = tid & 15u;
        const uint32_t row = row0 + r, col = col0 + ch * C;
        const bool ok = row < d.rows && col < d.cols;
        u32x4 raw = raws[pass];
        uint32_t flags;
        if constexpr (FMT == kMaskU8)
            flags = (C == 4) ? bytes4_to_bits(mlo[pass]) : (bytes4_to_bits(mlo[pass]) | (bytes4_to_bits(mhi[pass]) << 4));
        else
            flags = (C == 8) ? mlo[pass] : ((mlo[pass] >> (col & 4u)) & 0xFu);
        flags = ok ? flags : 0u;                 // everything of such a chunk is then masked to zero below
        uint32_t w4[4] = {raw.x, raw.y, raw.z, raw.w};
        if constexpr (DT == kF32) {
#pragma unroll
            for (int c = 0; c < 4; c++)
                w4[c] = ((flags >> c) & 1u) ? w4[c] : 0u;
            FN[r][ch] = (uint8_t)flags;
        } else {
#pragma unroll
            for (int c = 0; c < 4; c++) {
                const uint32_t keep_lo = ((flags >> (2 * c)) & 1u) ? 0x0000FFFFu : 0u;
                const uint32_t keep_hi = ((flags >> (2 * c + 1)) & 1u) ? 0xFFFF0000u : 0u;
                w4[c] &= keep_lo | keep_hi;
            }
            FN[r][ch] = (uint8_t)flags;
        }
        u32x4 mv = {w4[0], w4[1], w4[2], w4[3]};
        *(u32x4 *)&V[r][ch * C] = mv;
    }
    __syncthreads();

    // ---- E: compact.  Row units write W's values straight to memory (consecutive threads own
    // consecutive groups of a row); column units park W^T's values in LDS, column-major. ----
    {
        const size_t pitch = (size_t)(d.cols / M) * N;            // elements per row of vals
        const bool pair_ok = ES == 2 && ((N | (uint32_t)pitch) & 1u) == 0;
#pragma unroll
        for (int k = 0; k < NRU; k++) {
            const uint32_t u = tid + k * kThreads, r = u / GPT, g = u % GPT;
            if (u >= (uint32_t)(TR * GPT) || r >= r_valid || g >= g_valid)
                continue;   // outside the matrix: must not leave index bits in a row's padding
            uint32_t kb = 0;
            if constexpr (M >= C) {
#pragma unroll
                for (int q = 0; q < M / C; q++)
                    kb |= (uint32_t)FN[r][g * (M / C) + q] << (C * q);
            } else {
                kb = ((uint32_t)FN[r][g / (C / M)] >> (M * (g % (C / M)))) & ((1u << M) - 1u);
            }
            uint32_t sel, rem;
            choose_slots<M>(kb, N, sel, rem);
            T *dst = (T *)d.vals + (size_t)(row0 + r) * pitch + (size_t)(col0 / M + g) * N;
            unsigned long long code = 0, code_hi = 0;
            uint32_t pend = 0;
            if constexpr (NN != 0 && (NN * ES) % 16 == 0) {
                if ((((uintptr_t)d.vals | (pitch * ES)) & 15) == 0) {
                    // the group's NN values as whole 16-byte pieces
                    uint32_t out[NN * ES / 4];
#pragma unroll
                    for (int q = 0; q < NN * ES / 4; q++)
                        out[q] = 0;
#pragma unroll
                    for (int sl = 0; sl < NN; sl++) {
                        const uint32_t p = (uint32_t)__builtin_ctz(rem);
                        rem &= rem - 1u;
                        const uint32_t val = ((sel >> p) & 1u) ? (uint32_t)V[r][g * M + p] : 0u;
                        if constexpr (ES == 4)
                            out[sl] = val;
                        else
                            out[sl / 2] |= val << (16 * (sl & 1));
                        if (sl < HS)
                            code |= (unsigned long long)p << (sl * IB);
                        else
                            code_hi |= (unsigned long long)p << ((sl - HS) * IB);
                    }
#pragma unroll
                    for (int q = 0; q < NN * ES / 16; q++)
                        stream_store(u32x4{out[4 * q], out[4 * q + 1], out[4 * q + 2], out[4 * q + 3]}, (u32x4 *)dst + q);
                    if constexpr (SPLIT) {
                        put_code<HS * IB>(IDX[r], 2u * g, code);
                        put_code<HS * IB>(IDX[r], 2u * g + 1u, code_hi);
                    } else {
                        put_code<NN * IB>(IDX[r], g, code);
                    }
                    continue;
                }
            }
            if constexpr (M == 32)
                continue;   // not reached: the host sends 16:32 here only with vals aligned to 16 bytes
            for (uint32_t sl = 0; sl < N; sl++) {
                const uint32_t p = (uint32_t)__builtin_ctz(rem);
                rem &= rem - 1u;
                const uint32_t val = ((sel >> p) & 1u) ? (uint32_t)V[r][g * M + p] : 0u;
                if constexpr (ES == 4) {
                    ((uint32_t *)dst)[sl] = val;
                } else if (pair_ok) {
                    if (sl & 1u)
                        *(uint32_t *)(dst + sl - 1) = pend | (val << 16);
                    else
                        pend = val;
                } else {
                    dst[sl] = (T)val;
                }
                code |= (unsigned long long)p << (sl * IB);
            }
            lds_or_bits(IDX[r], g * N * IB, code);
        }
    }
#pragma unroll
    for (int k = 0; k < NCU; k++) {
        const uint32_t u = tid + k * kThreads, b = u / TC, c = u % TC;
        if (u >= (uint32_t)(BPT * TC) || b >= b_valid || c >= c_valid)
            continue;
        uint32_t kb = 0;
#pragma unroll
        for (int p = 0; p < M; p++)
            kb |= (((uint32_t)FN[b * M + p][c / C] >> (c % C)) & 1u) << p;
        uint32_t sel, rem;
        choose_slots<M>(kb, N, sel, rem);
        unsigned long long code = 0, code_hi = 0;
        if constexpr (NN != 0) {
#pragma unroll
            for (int sl = 0; sl < NN; sl++) {
                const uint32_t p = (uint32_t)__builtin_ctz(rem);
                rem &= rem - 1u;
                OT[c][b * NN + sl] = ((sel >> p) & 1u) ? V[b * M + p][c] : (T)0;
                if (sl < HS)
                    code |= (unsigned long long)p << (sl * IB);
                else
                    code_hi |= (unsigned long long)p << ((sl - HS) * IB);
            }
        } else {
            for (uint32_t sl = 0; sl < N; sl++) {
                const uint32_t p = (uint32_t)__builtin_ctz(rem);
                rem &= rem - 1u;
                OT[c][b * N + sl] = ((sel >> p) & 1u) ? V[b * M + p][c] : (T)0;
                code |= (unsigned long long)p << (sl * IB);
            }
        }
        if constexpr (SPLIT) {
            put_code<HS * IB>(IDXT[c], 2u * b, code);
            put_code<HS * IB>(IDXT[c], 2u * b + 1u, code_hi);
        } else if constexpr (NN != 0) {
            put_code<NN * IB>(IDXT[c], b, code);
        } else {
            lds_or_bits(IDXT[c], b * N * IB, code);
        }
    }
    __syncthreads();

    // ---- G: stream the staged W^T values and both index arrays out (row-per-lane-group, no divisions) ----
    {
        // valsT: c_valid rows (columns of W), b_valid*N elements each
        const uint32_t run = b_valid * N;
        const size_t pitch = (size_t)(d.rows / M) * N;
        T *dst = (T *)d.valsT + (size_t)col0 * pitch + (size_t)(row0 / M) * N;
        if (ES == 4 || (((run | (uint32_t)pitch | (uint32_t)((row0 / M) * N)) & 1u) == 0)) {
            // lanes per output row: a run has at most BPT * (M - 1) * ES / 4 dwords, BPT * M / 2 * ES / 4 when N = M/2
            constexpr uint32_t LWMAX = ES == 4 ? 64 : 32;
            constexpr uint32_t LW = (NN != 0 && 2 * NN == M) ? LWMAX / 2 : LWMAX;
            const uint32_t rd = run * ES / 4, x = tid % LW;
            if (x < rd)
                for (uint32_t c = tid / LW; c < c_valid; c += kThreads / LW)
                    stream_store(((const uint32_t *)&OT[c][0])[x], (uint32_t *)(dst + (size_t)c * pitch) + x);
        } else {
            for (uint32_t k = tid; k < c_valid * run; k += kThreads) {
                const uint32_t c = k / run, x = k - c * run;
                dst[(size_t)c * pitch + x] = OT[c][x];
            }
        }
    }
    {
        // idx: per row, the tile's bit string starts on a byte boundary (GPT*N*IB is a multiple of 8)
        constexpr uint32_t LW = IDXW * 4 <= 32 ? 32 : 64;
        const size_t pitch = ((size_t)(d.cols / M) * N * IB + 7) / 8;
        const uint32_t nbytes = (g_valid * N * IB + 7) / 8, x = tid % LW;
        unsigned char *dst = (unsigned char *)d.idx + (size_t)row0 * pitch + ((size_t)(col0 / M) * N * IB) / 8;
        if (x < nbytes)
            for (uint32_t r = tid / LW; r < r_valid; r += kThreads / LW)
                dst[(size_t)r * pitch + x] = ((const unsigned char *)&IDX[r][0])[x];
    }
    {
        constexpr uint32_t LW = IDXTW * 4 <= 32 ? 32 : 64;
        const size_t pitch = ((size_t)(d.rows / M) * N * IB + 7) / 8;
        const uint32_t nbytes = (b_valid * N * IB + 7) / 8, x = tid % LW;
        unsigned char *dst = (unsigned char *)d.idxT + (size_t)col0 * pitch + ((size_t)(row0 / M) * N * IB) / 8;
        if (x < nbytes)
            for (uint32_t c = tid / LW; c < c_valid; c += kThreads / LW)
                dst[(size_t)c * pitch + x] = ((const unsigned char *)&IDXT[c][0])[x];
    }
}

}  // namespace tmask

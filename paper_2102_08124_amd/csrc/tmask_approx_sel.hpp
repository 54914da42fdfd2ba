// Algorithm 1 (arXiv 2102.08124, Sec. 4) for bf16 weights with N = M/2, M in {8, 16}, as a
// threshold test on unique keys.
//
// In rank form an entry is kept iff at least K of its row precede it and at least K of its column
// do, in the (magnitude, row-major index) order.  A bf16 magnitude has 15 bits, so the order can be
// folded into one 32-bit key: |w| << 16 | j inside a row (fixed i, order by (|w|, j)) and
// |w| << 16 | i inside a column (order by (|w|, i)): exactly the tie-break of the sweep.  Keys of a
// line are distinct, hence "at least K = M/2 precede" <=> key >= t, where t is the N-th largest key of the
// line.  t comes from a small min/max network: sort both halves of the line, pair the i-th smallest
// of one half with the i-th largest of the other (the larger of each pair is in the upper half of
// the line), take the minimum of those.
//     keep(i,j) <=> rowkey(i,j) >= t_row(i)  and  colkey(i,j) >= t_col(j)
#pragma once
#include "tmask_device.hpp"
#include "tmask_networks.hpp"

namespace tmask {

// Same when the other half lives in the neighbouring lane (lane ^ 1): a = this lane's H keys.
template <int H>
__device__ __forceinline__ uint32_t upper_half_min_pair(uint32_t (&a)[H])
{
    sort_asc<H>(a);
    uint32_t t = 0xFFFFFFFFu;
#pragma unroll
    for (int i = 0; i < H; i++) {
        const uint32_t m = quad_xor_max<1>(a[i], a[H - 1 - i]);
        t = m < t ? m : t;
    }
    return t;
}

// Magnitude of column c (0..7) of a row held as four dwords, as the upper half of a 32-bit key.
__device__ __forceinline__ uint32_t bf16_mag_hi(const u32x4 &r, int c)
{
    const uint32_t d = (c >> 1) == 0 ? r.x : (c >> 1) == 1 ? r.y : (c >> 1) == 2 ? r.z : r.w;
    return (c & 1) ? (d & 0x7FFF0000u) : ((d << 16) & 0x7FFF0000u);
}

// bf16, M = 8 (one lane = one block) or M = 16 (two lanes = one block, 8 columns each).
// raw[i] = the 16 bytes (8 bf16) of row i of the lane's strip; gpos = lane's position in its block.
// Returns the kept magnitudes' sum; emit_row(i, b0, b1) receives the keep flags of row i as 0/1 bytes.
// Keys are built where they are used (column keys carry the row index, row keys the column index)
// so that only the raw rows stay live between the two passes.
// GENERAL: any number K of pruned entries per line, the same in every lane; the threshold is then the (K+1)-th
// smallest key of the line, read from the sorted line at a register index that is the same in every lane.  A row of
// sixteen lies in two lanes: each sorts its eight keys, takes the neighbour's sorted eight and merges the two runs.
template <int M, bool GENERAL = false, typename EmitRow>
__device__ __forceinline__ float approx_half_bf16(const u32x4 (&raw)[M], uint32_t gpos, EmitRow emit_row, uint32_t k_general = 0)
{
    const uint32_t kidx = GENERAL ? (__builtin_amdgcn_readfirstlane(k_general) & (uint32_t)(M - 1)) : 0u;
    constexpr int H = M / 2;
    // column thresholds: all M rows of a column are in the lane; key = |w| << 16 | i
    uint32_t tcol[8];
#pragma unroll
    for (int c = 0; c < 8; c++) {
        uint32_t a[H], b[H];
#pragma unroll
        for (int i = 0; i < H; i++) {
            a[i] = bf16_mag_hi(raw[i], c) | (uint32_t)i;
            b[i] = bf16_mag_hi(raw[H + i], c) | (uint32_t)(H + i);
        }
        if constexpr (GENERAL) {
            uint32_t srt[M];
#pragma unroll
            for (int i = 0; i < H; i++) {
                srt[i] = a[i];
                srt[H + i] = b[i];
            }
            sort_asc<M>(srt);
            tcol[c] = srt[kidx];
        } else {
            tcol[c] = upper_half_min<H>(a, b);
        }
        __builtin_amdgcn_sched_barrier(0);   // keep one column's network together: bounds register use
    }
    const uint32_t j0 = (M == 16) ? gpos * 8u : 0u;
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < M; i++) {
        // row threshold: key = |w| << 16 | j.  The row's dwords pass through an empty asm so that the
        // magnitudes are extracted again here instead of being kept in registers since the column pass.
        u32x4 r = raw[i];
        asm volatile("" : "+v"(r.x), "+v"(r.y), "+v"(r.z), "+v"(r.w));
        uint32_t mag[8], a[8];
#pragma unroll
        for (int c = 0; c < 8; c++) {
            mag[c] = bf16_mag_hi(r, c);
            a[c] = mag[c] | (j0 + (uint32_t)c);
        }
        uint32_t trow;
        if constexpr (GENERAL) {
            uint32_t srt[8];
#pragma unroll
            for (int c = 0; c < 8; c++)
                srt[c] = a[c];
            sort_asc<8>(srt);
            if constexpr (M == 8) {
                trow = srt[kidx];
            } else {
                uint32_t both[16];
#pragma unroll
                for (int c = 0; c < 8; c++) {
                    both[c] = srt[c];
                    both[8 + c] = quad_xor<1>(srt[c]);
                }
                merge_sorted8_asc(both);
                trow = both[kidx];
            }
        } else if constexpr (M == 8) {
            uint32_t lo[4] = {a[0], a[1], a[2], a[3]};
            uint32_t hi[4] = {a[4], a[5], a[6], a[7]};
            trow = upper_half_min<4>(lo, hi);
        } else {
            uint32_t srt[8];
#pragma unroll
            for (int c = 0; c < 8; c++)
                srt[c] = a[c];
            trow = upper_half_min_pair<8>(srt);
        }
        uint32_t bytes[2] = {0u, 0u};
#pragma unroll
        for (int c = 0; c < 8; c++) {
            const bool keep = (a[c] >= trow) & ((mag[c] | (uint32_t)i) >= tcol[c]);
            bytes[c >> 2] |= keep ? (1u << (8 * (c & 3))) : 0u;
            sum += keep ? __uint_as_float(mag[c]) : 0.f;
        }
        emit_row(i, bytes[0], bytes[1]);
        // the row's part of the sum is added here, not wherever the caller first needs the total (it would keep
        // every keep flag alive as a lane mask until then)
        asm volatile("" : "+v"(sum));
        __builtin_amdgcn_sched_barrier(0);   // finish (and store) a row before the next one starts
    }
    return sum;
}


// The row half alone (structured N:M pruning along rows at N = M/2): bit c of bits[i] = entry (i, c) of the lane's
// strip is among the N heaviest of its row group under the (magnitude, position) order.
// GENERAL (M = 8): any N, the threshold read from the sorted row group at index k_general = M - N.
template <int M, bool GENERAL = false>
__device__ __forceinline__ void row_half_keep_bf16(const u32x4 (&raw)[M], uint32_t gpos, uint32_t (&bits)[M],
                                                   uint32_t k_general = 0)
{
    static_assert(!GENERAL || M == 8, "a whole row group in one lane");
    const uint32_t kidx = GENERAL ? (__builtin_amdgcn_readfirstlane(k_general) & 7u) : 0u;
    const uint32_t j0 = (M == 16) ? gpos * 8u : 0u;
#pragma unroll
    for (int i = 0; i < M; i++) {
        uint32_t a[8];
#pragma unroll
        for (int c = 0; c < 8; c++)
            a[c] = bf16_mag_hi(raw[i], c) | (j0 + (uint32_t)c);
        uint32_t trow;
        if constexpr (GENERAL) {
            uint32_t srt[8];
#pragma unroll
            for (int c = 0; c < 8; c++)
                srt[c] = a[c];
            sort_asc<8>(srt);
            trow = srt[kidx];
        } else if constexpr (M == 8) {
            uint32_t lo[4] = {a[0], a[1], a[2], a[3]};
            uint32_t hi[4] = {a[4], a[5], a[6], a[7]};
            trow = upper_half_min<4>(lo, hi);
        } else {
            uint32_t srt[8];
#pragma unroll
            for (int c = 0; c < 8; c++)
                srt[c] = a[c];
            trow = upper_half_min_pair<8>(srt);
        }
        uint32_t b = 0;
#pragma unroll
        for (int c = 0; c < 8; c++)
            b |= (a[c] >= trow ? 1u : 0u) << c;
        bits[i] = b;
        __builtin_amdgcn_sched_barrier(0);   // one row at a time
    }
}

// =================================================================================================
// fp32, N = M/2, M = 8 or 16.  A 31-bit magnitude leaves no room for the index, so thresholds are
// taken on magnitudes alone: t = N-th largest of a line, u = (N+1)-th largest.  If t > u in every
// line of the strip, "key >= t" is exactly the rank test (no tie straddles the cut).  If some line has
// t == u the index order matters there; the caller then redoes the strip with approx_half_f32_ties (below).
// A line of a column (M rows) is lane-local; a line of a row is spread over G = M/4 lanes.
// =================================================================================================

// Both order statistics around the middle of 2H values held as two halves (sorted in place).
template <int H>
__device__ __forceinline__ void middle_pair(uint32_t (&a)[H], uint32_t (&b)[H], uint32_t &t, uint32_t &u)
{
    sort_asc<H>(a);
    sort_asc<H>(b);
    t = 0xFFFFFFFFu;
    u = 0u;
#pragma unroll
    for (int i = 0; i < H; i++) {
        const uint32_t x = a[i], y = b[H - 1 - i];
        const uint32_t hi = x > y ? x : y, lo = x > y ? y : x;
        t = hi < t ? hi : t;
        u = lo > u ? lo : u;
    }
}

template <>
__device__ __forceinline__ void middle_pair<4>(uint32_t (&a)[4], uint32_t (&b)[4], uint32_t &t, uint32_t &u)
{
    const uint32_t v[8] = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
    const Eight e = columns_of_8(v);
    t = fifth_of_8(e);
    u = fourth_of_8(e);
}

// Row of 8 over two lanes (4 values each): both lanes take the neighbour's four values and run the same network.
__device__ __forceinline__ void middle_pair_row8(uint32_t (&s)[4], uint32_t &t, uint32_t &u)
{
    const uint32_t v[8] = {s[0], s[1], s[2], s[3], quad_xor<1>(s[0]), quad_xor<1>(s[1]), quad_xor<1>(s[2]), quad_xor<1>(s[3])};
    const Eight e = columns_of_8(v);
    t = fifth_of_8(e);
    u = fourth_of_8(e);
}

// Row of 16 over four lanes (4 values each): merge lane pairs into sorted runs of 8, then split the
// two runs against each other.
__device__ __forceinline__ void middle_pair_row16(uint32_t (&s)[4], uint32_t gpos, uint32_t &t, uint32_t &u)
{
    sort_asc<4>(s);
    const bool upper = (gpos & 1u) != 0u;     // this lane keeps the larger half of its pair
    uint32_t m[4];
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const uint32_t hi = quad_xor_max<1>(s[i], s[3 - i]), lo = quad_xor_min<1>(s[i], s[3 - i]);
        m[i] = upper ? hi : lo;
    }
    // m is bitonic: two merge stages sort it
    cmpx(m[0], m[2]); cmpx(m[1], m[3]); cmpx(m[0], m[1]); cmpx(m[2], m[3]);
    uint32_t tl = 0xFFFFFFFFu, ul = 0u;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const uint32_t hi = quad_xor_max<3>(m[i], m[3 - i]), lo = quad_xor_min<3>(m[i], m[3 - i]);
        tl = hi < tl ? hi : tl;
        ul = lo > ul ? lo : ul;
    }
    t = quad_xor_min<1>(tl, tl);
    u = quad_xor_max<1>(ul, ul);
}

// a[i][c] = magnitude keys of the lane's strip (4 columns).  Fills bits[i] (bit c = keep) and the
// kept sum; returns true if some line had a tie across its cut (result then invalid).
// GENERAL (M = 8 only): any number K of pruned entries per line, the same in every lane: the line's eight keys are
// sorted, t = the (K+1)-th smallest and u = the K-th smallest are read at a register index that every lane shares.
template <int M, bool GENERAL = false>
__device__ __forceinline__ bool approx_half_f32(const uint32_t (&a)[M][4], uint32_t gpos, uint32_t (&rowbytes)[M],
                                                float &sum, uint32_t k_general = 0)
{
    static_assert(!GENERAL || M == 8, "a line of eight keys: one lane's column, two lanes' row");
    const uint32_t kidx = GENERAL ? (__builtin_amdgcn_readfirstlane(k_general) & 7u) : 0u;
    constexpr int H = M / 2;
    uint32_t tcol[4];
    bool tie = false;
#pragma unroll
    for (int c = 0; c < 4; c++) {
        uint32_t lo[H], hi[H], u;
#pragma unroll
        for (int i = 0; i < H; i++) {
            lo[i] = a[i][c];
            hi[i] = a[H + i][c];
        }
        if constexpr (GENERAL) {
            uint32_t srt[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            sort_asc<8>(srt);
            tcol[c] = srt[kidx];
            u = srt[(kidx - 1u) & 7u];
        } else {
            middle_pair<H>(lo, hi, tcol[c], u);
        }
        tie |= tcol[c] == u;
        __builtin_amdgcn_sched_barrier(0);
    }
    sum = 0.f;
#pragma unroll
    for (int i = 0; i < M; i++) {
        uint32_t s[4] = {a[i][0], a[i][1], a[i][2], a[i][3]};
        uint32_t trow, u;
        if constexpr (GENERAL) {
            uint32_t srt[8] = {s[0], s[1], s[2], s[3], quad_xor<1>(s[0]), quad_xor<1>(s[1]), quad_xor<1>(s[2]), quad_xor<1>(s[3])};
            sort_asc<8>(srt);
            trow = srt[kidx];
            u = srt[(kidx - 1u) & 7u];
        } else if constexpr (M == 8)
            middle_pair_row8(s, trow, u);
        else
            middle_pair_row16(s, gpos, trow, u);
        tie |= trow == u;
        uint32_t bytes = 0;
#pragma unroll
        for (int c = 0; c < 4; c++) {
            const bool keep = (a[i][c] >= trow) & (a[i][c] >= tcol[c]);
            bytes |= keep ? (1u << (8 * c)) : 0u;
            sum += keep ? __uint_as_float(a[i][c]) : 0.f;
        }
        rowbytes[i] = bytes;
        __builtin_amdgcn_sched_barrier(0);
    }
    return tie;
}

// The row half alone (N:M pruning along rows at N = M/2, fp32): bit c of bits[i] = entry (i, c) is at least the N-th
// largest magnitude of its row group.  Returns true if some group had a tie across its cut (result then invalid: the
// caller redoes the strip in the rank form).
template <int M>
__device__ __forceinline__ bool row_half_keep_f32(const uint32_t (&a)[M][4], uint32_t gpos, uint32_t (&bits)[M])
{
    bool tie = false;
#pragma unroll
    for (int i = 0; i < M; i++) {
        uint32_t s[4] = {a[i][0], a[i][1], a[i][2], a[i][3]};
        uint32_t trow, u;
        if constexpr (M == 8)
            middle_pair_row8(s, trow, u);
        else
            middle_pair_row16(s, gpos, trow, u);
        tie |= trow == u;
        uint32_t b = 0;
#pragma unroll
        for (int c = 0; c < 4; c++)
            b |= (a[i][c] >= trow ? 1u : 0u) << c;
        bits[i] = b;
    }
    return tie;
}

// The same result when some line has its cut among equal values: of the entries equal to the line's threshold t (the
// N-th largest value) the last N - #(entries above t) in position order stay, which is what the (magnitude, position)
// order of the sweep decides.  A column is lane-local; a row is spread over G = M/4 lanes, and an entry's share of the
// equal ones that stay is what the lanes to its right leave over.  About a quarter of the rank form's instructions.
template <int M>
__device__ __forceinline__ void approx_half_f32_ties(const uint32_t (&a_in)[M][4], uint32_t gpos, uint32_t (&rowbytes)[M],
                                                     float &sum)
{
    constexpr int H = M / 2, G = M / 4;
    constexpr uint32_t N = M / 2;
    // The keys pass through an empty asm: the thresholds are then worked out again here.  Otherwise the compiler reuses
    // the ones approx_half_f32 computed, which keeps all of them (and more) in registers on the way that has no ties:
    // 209 instead of 119 registers at M = 16, half the wavefronts per SIMD.
    uint32_t a[M][4];
#pragma unroll
    for (int i = 0; i < M; i++)
#pragma unroll
        for (int c = 0; c < 4; c++) {
            a[i][c] = a_in[i][c];
            asm volatile("" : "+v"(a[i][c]));
        }
    uint32_t colkeep[4];            // bit i: entry (i, c) stays as far as its column is concerned
#pragma unroll
    for (int c = 0; c < 4; c++) {
        uint32_t lo[H], hi[H], t, u;
#pragma unroll
        for (int i = 0; i < H; i++) {
            lo[i] = a[i][c];
            hi[i] = a[H + i][c];
        }
        middle_pair<H>(lo, hi, t, u);
        uint32_t gt = 0;
#pragma unroll
        for (int i = 0; i < M; i++)
            gt += a[i][c] > t ? 1u : 0u;
        uint32_t need = N - gt, w = 0;
#pragma unroll
        for (int i = M - 1; i >= 0; i--) {
            const bool take = a[i][c] == t && need != 0u;
            need -= take ? 1u : 0u;
            w |= ((a[i][c] > t || take) ? 1u : 0u) << i;
        }
        colkeep[c] = w;
        __builtin_amdgcn_sched_barrier(0);
    }
    sum = 0.f;
#pragma unroll
    for (int i = 0; i < M; i++) {
        uint32_t s[4] = {a[i][0], a[i][1], a[i][2], a[i][3]};
        uint32_t t, u;
        if constexpr (M == 8)
            middle_pair_row8(s, t, u);
        else
            middle_pair_row16(s, gpos, t, u);
        uint32_t gt = 0, eq = 0;
#pragma unroll
        for (int c = 0; c < 4; c++) {
            gt += a[i][c] > t ? 1u : 0u;
            eq += a[i][c] == t ? 1u : 0u;
        }
        // entries equal to t in the lanes to the right of this one (higher columns of the row)
        // (every cross-lane read happens with all lanes of the block enabled; only the use is conditional)
        uint32_t right;
        const uint32_t eq_next = quad_xor<1>(eq);
        if constexpr (G == 2) {
            gt += quad_xor<1>(gt);
            right = gpos == 0u ? eq_next : 0u;
        } else {
            gt += quad_xor<1>(gt);
            gt += quad_xor<2>(gt);
            const uint32_t pair_far = quad_xor<2>(eq + eq_next);
            right = ((gpos & 1u) ? 0u : eq_next) + (gpos < 2u ? pair_far : 0u);
        }
        const uint32_t stay = N - gt;                       // equal entries of the whole row that stay
        uint32_t need = stay > right ? stay - right : 0u;   // ... and of this lane, from its last column down
        uint32_t bytes = 0;
#pragma unroll
        for (int c = 3; c >= 0; c--) {
            const bool take = a[i][c] == t && need != 0u;
            need -= take ? 1u : 0u;
            const bool keep = (a[i][c] > t || take) && ((colkeep[c] >> i) & 1u);
            bytes |= keep ? (1u << (8 * c)) : 0u;
            sum += keep ? __uint_as_float(a[i][c]) : 0.f;
        }
        rowbytes[i] = bytes;
        __builtin_amdgcn_sched_barrier(0);
    }
}

}  // namespace tmask

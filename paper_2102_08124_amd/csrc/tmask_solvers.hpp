// Per-block solvers working on the strip layout (see tmask_device.hpp).
//   approx_keep   : Algorithm 1 of arXiv 2102.08124 (Sec. 4) in rank form
//   exact24_block : Eq. 3 optimum for 2:4 over all 90 feasible patterns (factored enumeration)
//   best_permutation4 : Eq. 3 optimum for 1:4 and 3:4 over the 24 permutations
//   exact_costs / exact_priced_start / exact_phases : the pieces of the Eq. 3 optimum for M = 8, 16 by successive
//                   shortest augmenting paths on the bipartite row/column network of Fig. 3 (put together in
//                   tmask_exact_balance.hpp)
#pragma once
#include "tmask_device.hpp"
#include "tmask_networks.hpp"

namespace tmask {

// =================================================================================================
// Algorithm 1 in rank form.
//
// Under the strict total order (magnitude key, then row-major index) the greedy sweep of
// Algorithm 1 -- take an entry while its row or its column has fewer than K taken entries --
// ends with exactly the entries that are among the K lightest of their row or of their column:
// the n-th lightest entry of a line (n <= K) meets fewer than K taken entries in that line when it
// is visited, and an entry outside the K lightest of both its lines finds both saturated.
// So  keep(i,j) <=> rank_in_row(i,j) >= K  and  rank_in_column(i,j) >= K,
// where rank = number of entries of the line that precede (i,j) in the order.  Because positions
// are static, "precedes" is `<=` against earlier positions and `<` against later ones.
// =================================================================================================

// rank bookkeeping for one ordered pair: `first` precedes `second` iff le.  Up to M = 8 the compare
// result stays a lane mask and feeds two add-with-carry instructions; at M = 16 that form costs
// registers and occupancy, plain 0/1 arithmetic is faster there.
template <int M>
__device__ __forceinline__ void rank_pair(bool le, uint32_t &r_first, uint32_t &r_second)
{
    if constexpr (M <= 8) {
        const lanemask_t m = lm(le);
        lm_inc(r_second, m);
        lm_inc(r_first, ~m);
    } else {
        const uint32_t v = le ? 1u : 0u;
        r_second += v;
        r_first += 1u - v;
    }
}

template <int M>
__device__ __forceinline__ void rank_one(bool precedes, uint32_t &r)
{
    if constexpr (M <= 8)
        lm_inc(r, lm(precedes));
    else
        r += precedes ? 1u : 0u;
}

// Column direction: all M rows of a column live in the lane.
// PIN: merge every flag into its row's bits at once.  Wanted at M = 16 when the flags are stored as bit masks:
// left alone the compiler carries all the compare results as lane masks to the place where the flags are
// stored (hundreds of spilled scalar registers, one wavefront per SIMD).  With byte masks the freer schedule is
// the faster one.
template <int M, int C, bool PIN = false>
__device__ __forceinline__ void col_rank_keep(const uint32_t (&a)[M][C], uint32_t K, uint32_t (&bits)[M])
{
#pragma unroll
    for (int i = 0; i < M; i++)
        bits[i] = 0;
#pragma unroll
    for (int c = 0; c < C; c++) {
        uint32_t r[M];
#pragma unroll
        for (int i = 0; i < M; i++)
            r[i] = 0;
#pragma unroll
        for (int i = 0; i < M; i++)
#pragma unroll
            for (int i2 = i + 1; i2 < M; i2++) {
                rank_pair<M>(a[i][c] <= a[i2][c], r[i], r[i2]);   // row i precedes row i2
            }
#pragma unroll
        for (int i = 0; i < M; i++) {
            bits[i] |= (r[i] >= K ? 1u : 0u) << c;
            if constexpr (PIN)
                asm volatile("" : "+v"(bits[i]));
        }
    }
}

// Row direction: a block-row is spread over G lanes (CL columns each); B blocks share a lane.
// gpos = position of the lane inside its group of G.  bits[i] &= row-keep.
template <int M, int C, int G, int B, bool PIN = false>
__device__ __forceinline__ void row_rank_keep(const uint32_t (&a)[M][C], uint32_t K, uint32_t gpos,
                                              uint32_t (&bits)[M])
{
    constexpr int CL = C / B;
#pragma unroll
    for (int i = 0; i < M; i++) {
        uint32_t keep = 0;
#pragma unroll
        for (int b = 0; b < B; b++) {
            uint32_t r[CL];
#pragma unroll
            for (int c = 0; c < CL; c++)
                r[c] = 0;
#pragma unroll
            for (int c = 0; c < CL; c++)
#pragma unroll
                for (int c2 = c + 1; c2 < CL; c2++) {
                    rank_pair<M>(a[i][b * CL + c] <= a[i][b * CL + c2], r[c], r[c2]);
                }
            if constexpr (G >= 2) {
                // keys are < 2^31, so "theirs <= mine" is "theirs < mine + 1"
                const uint32_t pb1 = ((gpos ^ 1u) < gpos) ? 1u : 0u;
#pragma unroll
                for (int c2 = 0; c2 < CL; c2++) {
                    const uint32_t t = quad_xor<1>(a[i][c2]);
#pragma unroll
                    for (int c = 0; c < CL; c++)
                        rank_one<M>(t < a[i][c] + pb1, r[c]);
                }
            }
            if constexpr (G == 4) {
                const uint32_t pb2 = ((gpos ^ 2u) < gpos) ? 1u : 0u;
                const uint32_t pb3 = ((gpos ^ 3u) < gpos) ? 1u : 0u;
#pragma unroll
                for (int c2 = 0; c2 < CL; c2++) {
                    const uint32_t t2 = quad_xor<2>(a[i][c2]);
                    const uint32_t t3 = quad_xor<3>(a[i][c2]);
#pragma unroll
                    for (int c = 0; c < CL; c++) {
                        rank_one<M>(t2 < a[i][c] + pb2, r[c]);
                        rank_one<M>(t3 < a[i][c] + pb3, r[c]);
                    }
                }
            }
#pragma unroll
            for (int c = 0; c < CL; c++)
                keep |= (r[c] >= K ? 1u : 0u) << (b * CL + c);
        }
        bits[i] &= keep;
        if constexpr (PIN)
            asm volatile("" : "+v"(bits[i]));
    }
}

template <int DT, int M, bool PIN = false>
__device__ __forceinline__ void approx_keep(const uint32_t (&a)[M][Geo<DT, M>::C], uint32_t K, uint32_t gpos,
                                            uint32_t (&bits)[M])
{
    using Ge = Geo<DT, M>;
    col_rank_keep<M, Ge::C, PIN>(a, K, bits);
    row_rank_keep<M, Ge::C, Ge::G, Ge::B, PIN>(a, K, gpos, bits);
}

// =================================================================================================
// Exact 2:4: all 0/1 4x4 matrices with two ones in every row and column (there are 90), fp32 sums.
// A row pattern is a pair of columns; pairs are numbered 0..5 = {01,02,03,12,13,23}.
// =================================================================================================

struct Patterns24 {
    uint8_t p[90][4];
    int n;
};

constexpr int kPairX[6] = {0, 0, 0, 1, 1, 2};
constexpr int kPairY[6] = {1, 2, 3, 2, 3, 3};

constexpr uint32_t pair_bits(int p) { return (1u << kPairX[p]) | (1u << kPairY[p]); }

constexpr Patterns24 make_patterns24()
{
    Patterns24 t{};
    t.n = 0;
    for (int p0 = 0; p0 < 6; p0++)
        for (int p1 = 0; p1 < 6; p1++)
            for (int p2 = 0; p2 < 6; p2++)
                for (int p3 = 0; p3 < 6; p3++) {
                    bool ok = true;
                    for (int c = 0; c < 4; c++) {
                        int s = ((pair_bits(p0) >> c) & 1) + ((pair_bits(p1) >> c) & 1) +
                                ((pair_bits(p2) >> c) & 1) + ((pair_bits(p3) >> c) & 1);
                        ok = ok && (s == 2);
                    }
                    if (ok) {
                        t.p[t.n][0] = (uint8_t)p0; t.p[t.n][1] = (uint8_t)p1;
                        t.p[t.n][2] = (uint8_t)p2; t.p[t.n][3] = (uint8_t)p3;
                        t.n++;
                    }
                }
    return t;
}

constexpr Patterns24 kPatterns24 = make_patterns24();
static_assert(kPatterns24.n == 90, "a 4x4 block has 90 feasible 2:4 transposable patterns");

constexpr uint32_t pattern_mask16(int k)
{
    return pair_bits(kPatterns24.p[k][0]) | (pair_bits(kPatterns24.p[k][1]) << 4) |
           (pair_bits(kPatterns24.p[k][2]) << 8) | (pair_bits(kPatterns24.p[k][3]) << 12);
}

// The 90 patterns factor through the column-count vector left by rows 0 and 1: a pattern is a pair
// (p0, p1) for rows 0,1 with column counts v, and a pair (p2, p3) for rows 2,3 with counts 2 - v.
// There are 19 such vectors (6 of type 2200 reached by one pair of pairs, 12 of type 2110 reached by
// two, 1 of type 1111 reached by six: 6*1*1 + 12*2*2 + 1*6*6 = 90), so the optimum is
//     max over v of  best01[v] + best23[2 - v],
// with best01 / best23 the best pair sums of the upper / lower two rows for each vector: 72 sums and
// 19 combinations instead of 90 four-term sums.
struct Halves24 {
    int vec_of[36];      // (p, q) -> index of the count vector of pair_bits(p) + pair_bits(q)
    int first_of[36];    // 1 if (p, q) is the first pair of pairs with that vector (enumeration order)
    int compl_of[19];    // index of the vector 2 - v
    int n_vec;
};

constexpr int count_code(int p, int q)
{
    int code = 0, mul = 1;
    for (int c = 0; c < 4; c++) {
        code += mul * (int)(((pair_bits(p) >> c) & 1u) + ((pair_bits(q) >> c) & 1u));
        mul *= 3;
    }
    return code;
}

constexpr Halves24 make_halves24()
{
    Halves24 h{};
    int codes[36] = {};
    h.n_vec = 0;
    for (int k = 0; k < 36; k++) {
        const int code = count_code(k / 6, k % 6);
        int idx = -1;
        for (int j = 0; j < h.n_vec; j++)
            if (codes[j] == code)
                idx = j;
        h.first_of[k] = idx < 0 ? 1 : 0;
        if (idx < 0) {
            idx = h.n_vec;
            codes[h.n_vec++] = code;
        }
        h.vec_of[k] = idx;
    }
    for (int j = 0; j < h.n_vec; j++) {
        const int want = 80 - codes[j];       // (2,2,2,2) in base 3 is 80; digits never borrow
        h.compl_of[j] = -1;
        for (int i = 0; i < h.n_vec; i++)
            if (codes[i] == want)
                h.compl_of[j] = i;
    }
    return h;
}

constexpr Halves24 kHalves24 = make_halves24();
static_assert(kHalves24.n_vec == 19, "rows 0,1 of a 2:4 pattern leave 19 possible column-count vectors");

// Best pair of row patterns per count vector for rows (r, r+1): value and 8-bit mask (row r in bits 0..3).
__device__ __forceinline__ void best_pairs24(const float (&pa)[6], const float (&pb)[6], float (&val)[19],
                                             uint32_t (&msk)[19])
{
#pragma unroll
    for (int k = 0; k < 36; k++) {
        const int idx = kHalves24.vec_of[k];
        const float s = pa[k / 6] + pb[k % 6];
        const uint32_t m = pair_bits(k / 6) | (pair_bits(k % 6) << 4);
        if (kHalves24.first_of[k]) {
            val[idx] = s;
            msk[idx] = m;
        } else {
            const bool better = s > val[idx];     // false for NaN: a feasible choice stays in place
            val[idx] = better ? s : val[idx];
            msk[idx] = better ? m : msk[idx];
        }
    }
}

// v[r][c] = |W| of one 4x4 block.  Returns the 16-bit keep mask (row r in bits 4r..4r+3) of an
// optimal pattern (the first one in a fixed evaluation order) and its kept sum in `best`.
__device__ __forceinline__ uint32_t exact24_block(const float (&v)[4][4], float &best)
{
    float ps[4][6];
#pragma unroll
    for (int r = 0; r < 4; r++)
#pragma unroll
        for (int p = 0; p < 6; p++)
            ps[r][p] = v[r][kPairX[p]] + v[r][kPairY[p]];
    float top[19], bot[19];
    uint32_t topm[19], botm[19];
    best_pairs24(ps[0], ps[1], top, topm);
    best_pairs24(ps[2], ps[3], bot, botm);
    uint32_t bm = 0;
#pragma unroll
    for (int j = 0; j < 19; j++) {
        const int jc = kHalves24.compl_of[j];
        const float s = top[j] + bot[jc];
        const uint32_t m = topm[j] | (botm[jc] << 8);
        if (j == 0) {
            best = s;
            bm = m;
        } else {
            const bool better = s > best;
            best = better ? s : best;
            bm = better ? m : bm;
        }
    }
    return bm;
}

// 1:4 and 3:4: one entry per row and per column is kept (1:4) or pruned (3:4), i.e. the pattern is one of the 24
// permutations.  v[r][c] = |W| of one 4x4 block.  Returns the 16-bit mask (row r in bits 4r..4r+3) of the permutation
// with the largest (LARGEST) or smallest sum, the first one in a fixed evaluation order, and that sum in `best`.  Rows
// 0 and 1 take an ordered pair of columns (12 ways); rows 2 and 3 share the two columns left and take the better of
// their two assignments.
template <bool LARGEST>
__device__ __forceinline__ uint32_t best_permutation4(const float (&v)[4][4], float &best)
{
    uint32_t bm = 0;
    bool first = true;
#pragma unroll
    for (int c0 = 0; c0 < 4; c0++)
#pragma unroll
        for (int c1 = 0; c1 < 4; c1++) {
            if (c1 == c0)
                continue;
            int x = -1, y = -1;
#pragma unroll
            for (int c = 0; c < 4; c++)
                if (c != c0 && c != c1) {
                    if (x < 0)
                        x = c;
                    else
                        y = c;
                }
            const float top = v[0][c0] + v[1][c1];
            const float b1 = v[2][x] + v[3][y], b2 = v[2][y] + v[3][x];
            const bool swap = LARGEST ? b2 > b1 : b2 < b1;
            const float s = top + (swap ? b2 : b1);
            const uint32_t m = (1u << c0) | (1u << (4 + c1)) |
                               (swap ? ((1u << (8 + y)) | (1u << (12 + x))) : ((1u << (8 + x)) | (1u << (12 + y))));
            const bool better = first || (LARGEST ? s > best : s < best);
            best = better ? s : best;
            bm = better ? m : bm;
            first = false;
        }
    return bm;
}

// =================================================================================================
// Exact, general (N, M): min-cost flow on the network of Fig. 3 (source -> rows, rows -> columns
// with unit capacity and cost |W_ij|, columns -> sink), solved by successive shortest paths.
//
// Costs are integers: c_ij = |W_ij| scaled by a power of two so that the block maximum lies in
// [2^(S-1), 2^S) and truncated.  Integer arithmetic makes every path sum exact, so the residual
// network never shows a negative cycle, label-correcting search converges, and the predecessor
// graph is a forest; truncation costs less than M*K*2^-(S-1) of the block maximum in retained L1
// (S = 27 for M <= 8, 26 for M = 16).
//
// Start: every column prunes the K rows that are lightest under row prices (exact_priced_start) -- a flow that
// saturates the column->sink edges and
// is cheapest among all flows with the same row imbalances.  Then, while some row has more than K
// pruned entries, find the cheapest alternating path from any such row to a row with fewer than K
// (row r -> column j through a pruned entry (r,j), column j -> row r' through an unpruned entry
// (r',j)) with a label-correcting search over row labels, and flip the entries along it.
//
// One block is held by G lanes, CL columns each; row labels are replicated in the G lanes and
// min-combined after each sweep, so all G lanes take the same decisions.
// =================================================================================================

constexpr int kInfDist = 0x70000000;   // unreachable label; kInfDist - 2^S is still above kReachable
constexpr int kReachable = 0x40000000; // every real label is below this: |label| <= (M-1) * 2^S < 2^30
constexpr uint32_t kNoPred = 0xFFFFFFFFu;

// r = lane-mask bit set ? a : b as exactly one v_cndmask (mask in a scalar register pair).
__device__ __forceinline__ uint32_t lm_pick(lanemask_t m, uint32_t a, uint32_t b)
{
    uint32_t r;
    asm("v_cndmask_b32_e64 %0, %1, %2, %3" : "=v"(r) : "v"(b), "v"(a), "s"(m));
    return r;
}

constexpr int exact_cost_bits(int M) { return (M == 16) ? 26 : 27; }

// |W| keys (fp32 bit patterns) of one block -> integer costs, see above.
template <int M, int CL, int G>
__device__ __forceinline__ void exact_costs(const uint32_t (&key)[M][CL], int (&cost)[M][CL])
{
    constexpr int S = exact_cost_bits(M);
    static_assert((M - 1) * (1ll << S) < kReachable, "labels must stay below the reachability threshold");
    // ---- integer costs ----
    uint32_t kmax = 0;
#pragma unroll
    for (int i = 0; i < M; i++)
#pragma unroll
        for (int c = 0; c < CL; c++)
            kmax = key[i][c] > kmax ? key[i][c] : kmax;
    if constexpr (G >= 2) {
        const uint32_t o = quad_xor<1>(kmax);
        kmax = o > kmax ? o : kmax;
    }
    if constexpr (G == 4) {
        const uint32_t o = quad_xor<2>(kmax);
        kmax = o > kmax ? o : kmax;
    }
    const uint32_t emax = (kmax >> 23) ? (kmax >> 23) : 1u;
#pragma unroll
    for (int i = 0; i < M; i++)
#pragma unroll
        for (int c = 0; c < CL; c++) {
            const uint32_t e = key[i][c] >> 23;
            const uint32_t mant = (key[i][c] & 0x7FFFFFu) | (e ? 0x800000u : 0u);
            const uint32_t sh = emax - (e ? e : 1u);
            cost[i][c] = sh < 32u ? (int)((mant << (S - 24)) >> sh) : 0;
        }

}

// Pruned entries per row, identical in the G lanes of the block.
template <int M, int CL, int G>
__device__ __forceinline__ void exact_counts(const uint32_t (&xcol)[CL], uint32_t (&cnt)[M])
{
#pragma unroll
    for (int i = 0; i < M; i++) {
        uint32_t n = 0;
#pragma unroll
        for (int c = 0; c < CL; c++)
            n += (xcol[c] >> i) & 1u;
        if constexpr (G >= 2)
            n += quad_xor<1>(n);
        if constexpr (G == 4)
            n += quad_xor<2>(n);
        cnt[i] = n;
    }
}

// Start for N = M/2 with row prices: column c prunes the K rows with the smallest cost + price (ties: lower
// row first).  Whatever the prices, the result is the cheapest pruning for the row counts it has: the price
// term of any pruning with those counts is the same sum over rows of price x count, so being cheapest under
// cost + price means being cheapest under cost alone.  That is all the augmenting searches ask of their
// start, so prices can even out the row counts before the first search: a row with too many pruned entries
// becomes dearer to prune, one with too few cheaper, every column chooses again, in rounds with a shrinking
// step: at M = 8 twelve rounds, first step 3/64 .. 3/32 of the largest cost, times 11/16 per round; at M = 16
// twenty rounds, first step 1/32 .. 1/16 of the largest cost, times 3/4 per round (both settled by timing on
// the device).  The prices of the round with the smallest total excess are kept; xcol is that round's choice
// and the return value its excess.  On random blocks the searches that follow drop from 3.1 per block (no
// prices) to 0.2 at M = 8 and from 6.3 to well under 0.5 at M = 16; a round costs about a third of one sweep of
// a search and runs with every lane busy, where the searches keep 40-50 % of the lanes busy.
//
// Keys are (cost + price + 2^(S-1)) << 4 | tie-break with |price| < 2^(S-1): below 2^(S+5) <= 2^32 for costs < 2^S.
// The tie-break of entry (i, j) is (i - j) mod M, not the row alone: columns with equal costs (blocks of an
// unstructured-sparse matrix are full of zeros) then prune different rows, a band, instead of all the same ones,
// which no row price could tell apart (4096^2 fp32 with 90 % zeros: 4:8 270 -> 146 us, 8:16 931 -> 370 us; all zeros:
// 181 -> 57 us, 544 -> 120 us).
// Prices are held unshifted (the shift rides on the add that forms a key); the step times the count is a 24-bit
// multiply-add (step < 2^23, counts <= M), the full 32-bit multiply runs at a quarter of the rate; the excess is
// taken as half the sum of |count - K| (the counts of a block always add up to M*K), one instruction per row.
// GENERAL: any 0 < K < M, the same in every lane (the threshold then comes from a full sort of the column's keys and a
// register read at that index; 24 instead of 12 instructions at M = 8, 91 instead of 60 at M = 16); otherwise K = M/2.
template <int M, int CL, int G, bool GENERAL = false>
__device__ __forceinline__ uint32_t exact_priced_start(const int (&cost)[M][CL], uint32_t gpos, uint32_t (&xcol)[CL],
                                                       uint32_t k_general = 0)
{
    constexpr int H = M / 2;
    const int K = GENERAL ? (int)__builtin_amdgcn_readfirstlane(k_general) : M / 2;
    constexpr int S = exact_cost_bits(M);
    constexpr int ROUNDS = (M == 16) ? 20 : 12;
    constexpr int PMIN = 1, PMAX = (1 << S) - 1;                // price + 2^(S-1)
    uint32_t ck[M][CL];
    int pr[M], best_pr[M];                                      // price + 2^(S-1)
#pragma unroll
    for (int i = 0; i < M; i++) {
        pr[i] = 1 << (S - 1);
#pragma unroll
        for (int c = 0; c < CL; c++)
            ck[i][c] = ((uint32_t)cost[i][c] << 4) | (((uint32_t)i - (gpos * (uint32_t)CL + (uint32_t)c)) & (uint32_t)(M - 1));
    }
    // the column's threshold key under the prices p: the K pruned rows are the keys below it
    auto threshold = [&](int c, const int (&p)[M], uint32_t (&k)[M]) {
        uint32_t lo[H], hi[H];
#pragma unroll
        for (int i = 0; i < M; i++)
            k[i] = ((uint32_t)p[i] << 4) + ck[i][c];
#pragma unroll
        for (int i = 0; i < H; i++) {
            lo[i] = k[i];
            hi[i] = k[H + i];
        }
        if constexpr (GENERAL) {
            uint32_t srt[M];
#pragma unroll
            for (int i = 0; i < M; i++)
                srt[i] = k[i];
            sort_asc<M>(srt);
            return srt[(uint32_t)K & (uint32_t)(M - 1)];      // the (K+1)-th smallest; the index is the same in every lane
        } else {
            return upper_half_min<H>(lo, hi);
        }
    };
    int step = (M == 16) ? (4 << (S - 7)) : (3 << (S - 6));
    static_assert(((M == 16) ? (4 << (S - 7)) : (3 << (S - 6))) < (1 << 23), "the step is an operand of a 24-bit multiply");
    uint32_t best = 0xFFFFFFFFu;                                 // twice the excess
#pragma unroll 1
    for (int round = 0; round <= ROUNDS; round++) {
        uint32_t n[M];
#pragma unroll
        for (int i = 0; i < M; i++)
            n[i] = 0;
#pragma unroll
        for (int c = 0; c < CL; c++) {
            uint32_t k[M];
            const uint32_t t = threshold(c, pr, k);
#pragma unroll
            for (int i = 0; i < M; i++)
                lm_inc(n[i], lm(k[i] < t));
            if constexpr (CL > 4)
                __builtin_amdgcn_sched_barrier(0);   // one column at a time: interleaving them costs M registers each
        }
        uint32_t e2 = 0;
#pragma unroll
        for (int i = 0; i < M; i++) {
            if constexpr (G >= 2)
                n[i] = quad_xor_sum<1>(n[i]);
            if constexpr (G == 4)
                n[i] = quad_xor_sum<2>(n[i]);
            e2 = __builtin_amdgcn_sad_u8(n[i], (uint32_t)K, e2);      // counts are below 256: |n - K| of the low byte
        }
        const bool better = e2 < best;
        best = better ? e2 : best;
        const int back = step * K;
#pragma unroll
        for (int i = 0; i < M; i++) {
            best_pr[i] = better ? pr[i] : best_pr[i];
            const int p = __mul24(step, (int)n[i]) + pr[i] - back;
            pr[i] = p > PMAX ? PMAX : p < PMIN ? PMIN : p;
        }
        step = (step * (M == 16 ? 12 : 11)) >> 4;
    }
#pragma unroll
    for (int c = 0; c < CL; c++) {
        uint32_t k[M];
        const uint32_t t = threshold(c, best_pr, k);
        uint32_t x = 0;
#pragma unroll
        for (int i = 0; i < M; i++)
            x |= (k[i] < t ? 1u : 0u) << i;
        xcol[c] = x;
    }
    return best >> 1;
}

// Up to max_phases searches, each followed by its augmentations; cnt is kept up to date.  Returns true when
// every row has exactly K pruned entries (always after at most M*M searches).
template <int M, int CL, int G>
__device__ __forceinline__ bool exact_phases(const int (&cost)[M][CL], uint32_t K, uint32_t gpos, uint32_t (&xcol)[CL],
                                             uint32_t (&cnt)[M], int max_phases)
{
    uint32_t rowid[M];   // row numbers in registers, operands of the selects below
#pragma unroll
    for (int i = 0; i < M; i++)
        rowid[i] = (uint32_t)i;

    // ---- augment until every row has exactly K pruned ----
    for (int phase = 0; phase < max_phases; phase++) {
        int drow[M];
        uint32_t prow[M];
        lanemask_t any_excess = 0;
        uint32_t deficit = 0;
#pragma unroll
        for (int i = 0; i < M; i++) {
            const lanemask_t ex = lm(cnt[i] > K);
            any_excess |= ex;
            deficit |= (cnt[i] < K ? 1u : 0u) << i;
            drow[i] = (int)lm_pick(ex, 0u, (uint32_t)kInfDist);
            prow[i] = kNoPred;
        }
        if (!lm_test(any_excess))
            return true;

        // label-correcting sweeps over the columns
        lanemask_t changed;
        int sweeps = 0;
        do {
            changed = 0;
#pragma unroll
            for (int c = 0; c < CL; c++) {
                lanemask_t pm[M];            // row i is pruned in this column
#pragma unroll
                for (int i = 0; i < M; i++)
                    pm[i] = lm((xcol[c] & (1u << i)) != 0u);
                // cheapest way to reach the column: through a pruned entry of a reached row
                uint32_t dcol = (uint32_t)kInfDist, from = 0;
#pragma unroll
                for (int i = 0; i < M; i++) {
                    const int t = drow[i] - cost[i][c];
                    const lanemask_t better = pm[i] & lm(t < (int)dcol);
                    dcol = lm_pick(better, (uint32_t)t, dcol);
                    from = lm_pick(better, rowid[i], from);
                }
                // an unreachable column must not improve anything: kInfDist + cost >= every label
                dcol = lm_pick(lm((int)dcol < kReachable), dcol, (uint32_t)kInfDist);
                const uint32_t code = ((gpos * CL + c) << 4) | from;
                // leave the column through its unpruned entries
#pragma unroll
                for (int i = 0; i < M; i++) {
                    const int t = (int)dcol + cost[i][c];
                    const lanemask_t better = ~pm[i] & lm(t < drow[i]);
                    drow[i] = (int)lm_pick(better, (uint32_t)t, (uint32_t)drow[i]);
                    prow[i] = lm_pick(better, code, prow[i]);
                    changed |= better;
                }
            }
            uint32_t chg = lm_test(changed) ? 1u : 0u;
            if constexpr (G >= 2) {
                const bool before = (gpos ^ 1u) < gpos;
#pragma unroll
                for (int i = 0; i < M; i++) {
                    const int od = (int)quad_xor<1>((uint32_t)drow[i]);
                    const uint32_t op = quad_xor<1>(prow[i]);
                    const bool take = (od < drow[i]) || (od == drow[i] && before);
                    drow[i] = take ? od : drow[i];
                    prow[i] = take ? op : prow[i];
                }
                chg |= quad_xor<1>(chg);
            }
            if constexpr (G == 4) {
                const bool before = (gpos ^ 2u) < gpos;
#pragma unroll
                for (int i = 0; i < M; i++) {
                    const int od = (int)quad_xor<2>((uint32_t)drow[i]);
                    const uint32_t op = quad_xor<2>(prow[i]);
                    const bool take = (od < drow[i]) || (od == drow[i] && before);
                    drow[i] = take ? od : drow[i];
                    prow[i] = take ? op : prow[i];
                }
                chg |= quad_xor<2>(chg);
            }
            changed = lm(chg != 0u);
            sweeps++;
        } while (lm_test(changed) && sweeps <= M);

        // At convergence every predecessor edge is tight (label of the head = label of the tail + edge cost), so
        // flipping along ANY predecessor chain keeps the reduced costs of the residual network non-negative:
        // the pruning stays cheapest for its row imbalances.  One search therefore serves several augmentations:
        // every reachable row that lacks pruned entries takes its chain, as long as the chains use different
        // columns and different rows (a row with excess may end several chains while its excess lasts).
        uint32_t cand = 0;
#pragma unroll
        for (int i = 0; i < M; i++)
            cand |= (((deficit >> i) & 1u) && drow[i] < kReachable ? 1u : 0u) << i;
        if (cand == 0u)
            break;   // cannot happen for 0 < K < M; guards against looping on corrupt state
        uint32_t used_rows = 0, used_cols = 0;
        while (cand) {
            const uint32_t target = (uint32_t)__builtin_ctz(cand);
            cand &= cand - 1u;
            // first walk: which rows and columns does the chain use, and where does it end
            uint32_t r = target, rows = 0, cols = 0;
            bool ended = false;
            for (int step = 0; step < M; step++) {
                uint32_t pp = kNoPred;
#pragma unroll
                for (int i = 0; i < M; i++)
                    pp = (r == (uint32_t)i) ? prow[i] : pp;
                if (pp == kNoPred) {
                    ended = true;
                    break;
                }
                rows |= 1u << r;
                cols |= 1u << (pp >> 4);
                r = pp & 15u;
            }
            uint32_t src_cnt = 0;
#pragma unroll
            for (int i = 0; i < M; i++)
                src_cnt = (r == (uint32_t)i) ? cnt[i] : src_cnt;
            const bool ok = ended && (rows & used_rows) == 0u && (cols & used_cols) == 0u &&
                            ((used_rows >> r) & 1u) == 0u && src_cnt > K;
            if (!ok)
                continue;   // left for the next search
            used_rows |= rows;
            used_cols |= cols;
            // second walk: flip the entries along the chain back to the row with excess
            const uint32_t src = r;
            r = target;
            for (int step = 0; step < M; step++) {
                uint32_t pp = kNoPred;
#pragma unroll
                for (int i = 0; i < M; i++)
                    pp = (r == (uint32_t)i) ? prow[i] : pp;
                if (pp == kNoPred)
                    break;
                const uint32_t j = pp >> 4, f = pp & 15u;
#pragma unroll
                for (int c = 0; c < CL; c++)
                    if (j == gpos * CL + c)
                        xcol[c] ^= (1u << r) | (1u << f);
                r = f;
            }
            // the chain's end loses one pruned entry, the target gains one
#pragma unroll
            for (int i = 0; i < M; i++)
                cnt[i] += (target == (uint32_t)i ? 1u : 0u) - (src == (uint32_t)i ? 1u : 0u);
        }
    }
    bool excess = false;
#pragma unroll
    for (int i = 0; i < M; i++)
        excess |= cnt[i] > K;
    return !excess;
}

}  // namespace tmask

// tmask: the column-per-lane kernels.  They serve (a) M = 32 for every entry point (the compression at 16:32 of aligned
// matrices excepted: the tiled pack kernel takes it), (b) M = 4, 8, 16 when a matrix
// misses the 16-byte alignment the strip kernels read with (only the method's own requirement is left: rows and cols
// multiples of M, the masks being defined per M x M block; arXiv 2102.08124, Sec. 4) and (c) Algorithm 1 and row
// pruning with N != M/2 at M = 16, where the strip kernels have only their rank form (Algorithm 1 at bf16 excepted: it
// has a threshold form on the strips).  gfx950 only.
//
// Layout.  A workgroup is one wavefront and works through tiles of M rows x 64 columns: lane l holds column l of the
// tile, all M rows, in registers, read and written element by element (no alignment needed).  A block is the M
// neighbouring lanes [b*M, b*M + M); the wavefront holds 64 / M blocks side by side.  Column-direction work is
// lane-local; for row-direction work the block is transposed through LDS (pitch M + 1 words, conflict-free), so that
// lane j of a block holds row j, and the answer travels back as one bit word per row.  Yes/no facts about a row of
// the block are also read off a wavefront ballot: bits [b*M, b*M + M) of ballot(flag of row i) are row i of block b.
//
// The mask and exact kernels are bound by the vector ALU (a threshold from a sorting network per line of M keys and,
// for the exact solver, per price round; the index arithmetic of staging, compaction and copy-out in the pack
// kernel), none of them by HBM.
#include <hip/hip_runtime.h>

#include <cstring>

#include "../../include/tmask.h"
#include "tmask_device.hpp"
#include "tmask_host.hpp"
#include "tmask_networks.hpp"

namespace tmask {

constexpr int kCwThreads = 64;
constexpr int kMaxCwBatch = 224;

struct CwMat {
    const void *w;
    void *mask;          // output of the mask kernels (may be null for the dense one-pass calls), input of score / pack
    void *aux;           // mask kernels: dense output (or null); score: per-block objective of this matrix (or null)
    uint32_t ld, mask_ld, ld_aux, cols;
    uint32_t tpr;        // tiles per block-row = ceil(cols / 64)
    uint32_t n_tiles;    // tpr * rows / M
    uint32_t wg0, n_wg;  // first workgroup of this matrix in the launch, and how many it has (each strides over tiles)
    uint32_t div_mul, div_shift;   // t / tpr
};

struct CwArgs {
    CwMat m[kMaxCwBatch];
    uint32_t n, K, N, partial0;
    void *partials;
};
static_assert(sizeof(CwArgs) <= 16384, "descriptor table is sized to stay a small kernel argument");

__device__ __forceinline__ int cw_find(const CwArgs &a, uint32_t wg)
{
    int lo = 0, hi = (int)a.n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (a.m[mid].wg0 <= wg)
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo;
}

template <int DT>
__device__ __forceinline__ uint32_t cw_load(const void *w, size_t idx)
{
    if constexpr (DT == kF32)
        return __builtin_nontemporal_load((const uint32_t *)w + idx);
    else
        return (uint32_t)__builtin_nontemporal_load((const uint16_t *)w + idx);
}

template <int DT>
__device__ __forceinline__ void cw_store(void *w, size_t idx, uint32_t v)
{
    if constexpr (DT == kF32)
        ((uint32_t *)w)[idx] = v;
    else
        ((uint16_t *)w)[idx] = (uint16_t)v;
}

// |W| as an fp32 bit pattern: the ordering key, and (as a float) the magnitude itself
template <int DT>
__device__ __forceinline__ uint32_t cw_key(uint32_t raw)
{
    return DT == kF32 ? (raw & 0x7FFFFFFFu) : ((raw << 16) & 0x7FFF0000u);
}

template <int M>
__device__ __forceinline__ uint32_t seg_mask()
{
    return (uint32_t)((1ull << M) - 1ull);
}

// bits [blk*M, blk*M + M) of a wavefront ballot
template <int M>
__device__ __forceinline__ uint32_t seg_of(lanemask_t b, uint32_t blk)
{
    return (uint32_t)(b >> (blk * M)) & seg_mask<M>();
}

// sum / max over the M lanes of a block (butterfly, fixed order: deterministic)
template <int M>
__device__ __forceinline__ float seg_sum(float v)
{
#pragma unroll
    for (int off = M / 2; off >= 1; off >>= 1)
        v += __shfl_xor(v, off, 64);
    return v;
}

template <int M>
__device__ __forceinline__ uint32_t seg_max(uint32_t v)
{
#pragma unroll
    for (int off = M / 2; off >= 1; off >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)v, off, 64);
        v = o > v ? o : v;
    }
    return v;
}

struct CwTile {
    uint32_t br, col0, col;   // block-row, first column of the tile (both the same in every lane), the lane's column
    bool active;
};

// Tile t of a matrix.  ADJ > 1 (used where a workgroup takes exactly one tile): workgroups go to the eight XCDs
// round-robin, and a tile row of 64 mask bytes is half a cache line, so neighbouring tiles are renumbered to meet on
// one XCD (workgroup t -> tile ((k / ADJ) * 8 + q) * ADJ + k % ADJ with q = t % 8, k = t / 8) instead of each
// fetching or partly writing the line: 8192^2 fp32 16:32 score 63 -> 56 us, Algorithm 1 73 -> 71 us, with the masked
// copy 144 -> 132 us; row pruning loses (65 -> 69 us) and keeps the plain order; bf16 is indifferent.
template <uint32_t ADJ = 1>
__device__ __forceinline__ CwTile cw_tile(const CwMat &md, uint32_t t)
{
    CwTile p;
    if constexpr (ADJ > 1) {
        const uint32_t full = md.n_tiles / (8u * ADJ) * (8u * ADJ);
        if (md.n_wg == md.n_tiles && t < full) {
            const uint32_t q = t & 7u, k = t >> 3;
            t = ((k / ADJ) * 8u + q) * ADJ + (k % ADJ);
        }
    }
    p.br = (uint32_t)(((uint64_t)t * md.div_mul) >> md.div_shift);
    p.col0 = (t - p.br * md.tpr) * 64u;
    p.col = p.col0 + threadIdx.x;
    p.active = p.col < md.cols;
    return p;
}

// The lane's column of the tile, M rows.  A row of the tile starts at an address that is the same in every lane (it
// advances in scalar registers), the lane adds its own column: one load instruction per row and nothing else.
template <int DT, int M>
__device__ __forceinline__ void cw_load_column(const CwMat &md, const CwTile &p, uint32_t (&raw)[M])
{
    constexpr size_t ES = DT == kF32 ? 4 : 2;
    const char *row = (const char *)md.w + ((size_t)p.br * M * md.ld + p.col0) * ES;
    const size_t pitch = (size_t)md.ld * ES;
#pragma unroll
    for (int i = 0; i < M; i++)
        raw[i] = 0u;
    if (p.active) {
#pragma unroll
        for (int i = 0; i < M; i++) {
            if constexpr (DT == kF32)
                raw[i] = __builtin_nontemporal_load((const uint32_t *)row + threadIdx.x);
            else
                raw[i] = (uint32_t)__builtin_nontemporal_load((const uint16_t *)row + threadIdx.x);
            row += pitch;
        }
    }
}

// the (K+1)-th smallest of M keys (1 <= K <= M - 1; the keys may repeat).  M = 32: two halves of 16 sorted by network,
// for K = 16 the minimum over i of max(a_i, b_15-i), for any other K a bitonic merge and a register read at an index
// that is the same in every lane.  M <= 16: one sorting network and that register read.
template <int M>
__device__ __forceinline__ uint32_t cw_threshold(const uint32_t (&k)[M], uint32_t K)
{
    if constexpr (M == 32) {
        uint32_t a[16], b[16];
#pragma unroll
        for (int i = 0; i < 16; i++) {
            a[i] = k[i];
            b[i] = k[16 + i];
        }
        sort_asc<16>(a);
        sort_asc<16>(b);
        uint32_t t;
        if (K == 16u) {
            t = 0xFFFFFFFFu;
#pragma unroll
            for (int i = 0; i < 16; i++) {
                const uint32_t m = a[i] > b[15 - i] ? a[i] : b[15 - i];
                t = m < t ? m : t;
            }
        } else {
            uint32_t s[32];
#pragma unroll
            for (int i = 0; i < 16; i++) {
                s[i] = a[i];
                s[16 + i] = b[15 - i];
            }
            bitonic_merge_asc<32>(s);
            t = s[__builtin_amdgcn_readfirstlane(K) & 31u];
        }
        return t;
    } else {
        uint32_t s[M];
#pragma unroll
        for (int i = 0; i < M; i++)
            s[i] = k[i];
        sort_asc<M>(s);
        return s[__builtin_amdgcn_readfirstlane(K) & (uint32_t)(M - 1)];
    }
}

// M magnitudes held by one lane: bit i of the result is set when entry i is among the first K of the (magnitude,
// position) order, i.e. pruned: the entries below the (K+1)-th smallest key.  bf16 keys carry the position in their low
// bits (15 + 5 bits), so they are distinct.  fp32 magnitudes are compared as they are; if the threshold value occurs
// on both sides of the cut, fewer than K entries lie below it and the missing ones are the entries equal to it at the
// lowest positions (a wavefront-uniform detour).  At M = 32: 350-550 instructions against 1500 for pairwise ranks.
template <int DT, int M>
__device__ __forceinline__ uint32_t cw_pruned(const uint32_t (&mag)[M], uint32_t K)
{
    uint32_t k[M];
#pragma unroll
    for (int i = 0; i < M; i++)
        k[i] = DT == kF32 ? mag[i] : ((mag[i] >> 11) | (uint32_t)i);
    const uint32_t t = cw_threshold<M>(k, K);
    uint32_t w = 0;
#pragma unroll
    for (int i = M - 1; i >= 0; i--)
        lm_shift_in(w, lm(k[i] < t));
    if constexpr (DT == kF32) {
        const uint32_t lt = (uint32_t)__builtin_popcount(w);
        if (lm(lt != K) != 0) {
            uint32_t eq = 0;
#pragma unroll
            for (int i = M - 1; i >= 0; i--)
                lm_shift_in(eq, lm(k[i] == t));
            uint32_t q = K - lt;
            while (lm(q != 0u) != 0) {
                const uint32_t low = q != 0u ? (eq & (0u - eq)) : 0u;
                w |= low;
                eq ^= low;
                q -= q != 0u ? 1u : 0u;
            }
        }
    }
    return w;
}

// An M x M bit matrix held as one word per lane by the M lanes of a block (lane l, bit i) -> its transpose (lane i,
// bit l): log2 M rounds of swapping the off-diagonal quarters at sizes M/2, ..., 1 with the lane that far away.
template <int M>
__device__ __forceinline__ uint32_t cw_transpose(uint32_t w)
{
#pragma unroll
    for (int s = M / 2; s >= 1; s >>= 1) {
        const uint32_t m = s == 16 ? 0x0000FFFFu : s == 8 ? 0x00FF00FFu : s == 4 ? 0x0F0F0F0Fu : s == 2 ? 0x33333333u : 0x55555555u;
        const uint32_t o = (uint32_t)__shfl_xor((int)w, s, 64);
        w = (threadIdx.x & (uint32_t)s) ? ((w & ~m) | ((o >> s) & m)) : ((w & m) | ((o << s) & ~m));
    }
    return w;
}

template <int M>
__device__ __forceinline__ uint32_t seg_sum_u32(uint32_t v)
{
#pragma unroll
    for (int off = M / 2; off >= 1; off >>= 1)
        v += (uint32_t)__shfl_xor((int)v, off, 64);
    return v;
}

// Writes the keep flags of the lane's column (bit i of `keep` = row i) as mask entries.
template <int M, int FMT>
__device__ __forceinline__ void cw_store_mask(const CwMat &md, const CwTile &p, uint32_t keep)
{
    if constexpr (FMT == kMaskU8) {
        if (p.active) {
            unsigned char *row = (unsigned char *)md.mask + (size_t)p.br * M * md.mask_ld + p.col0;   // same in every lane
#pragma unroll
            for (int i = 0; i < M; i++) {
                row[threadIdx.x] = (unsigned char)((keep >> i) & 1u);
                row += md.mask_ld;
            }
        }
    } else {
        // the 64 flags of a row are a ballot; lanes 0..7 each store one of its bytes (cols is a multiple of 8)
        const uint32_t lane = threadIdx.x;
        const uint32_t col0 = p.col - lane;
        unsigned char *mb = (unsigned char *)md.mask + (size_t)p.br * M * md.mask_ld + (col0 >> 3) + lane;
        const bool writer = lane < 8u && col0 + lane * 8u < md.cols;
#pragma unroll
        for (int i = 0; i < M; i++) {
            const lanemask_t b = lm(p.active && ((keep >> i) & 1u));
            if (writer)
                mb[(size_t)i * md.mask_ld] = (unsigned char)(b >> (lane * 8u));
        }
    }
}

// Reads the mask entries of the lane's column into bit i = row i.
template <int M, int FMT>
__device__ __forceinline__ uint32_t cw_load_mask(const CwMat &md, const CwTile &p)
{
    uint32_t bits = 0;
    if (p.active) {
        if constexpr (FMT == kMaskU8) {
            const unsigned char *row = (const unsigned char *)md.mask + (size_t)p.br * M * md.mask_ld + p.col0;
#pragma unroll
            for (int i = 0; i < M; i++) {
                bits |= (row[threadIdx.x] != 0 ? 1u : 0u) << i;
                row += md.mask_ld;
            }
        } else {
            const unsigned char *mb = (const unsigned char *)md.mask + (size_t)p.br * M * md.mask_ld + (p.col >> 3);
#pragma unroll
            for (int i = 0; i < M; i++)
                bits |= (((uint32_t)mb[(size_t)i * md.mask_ld] >> (p.col & 7u)) & 1u) << i;
        }
    }
    return bits;
}

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f)
{
    const uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u)
        return (u >> 16) | 0x0040u;                      // NaN stays NaN
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// =====================================================================================================================
// Algorithm 1 (rank form), row pruning, and their dense one-pass forms
// =====================================================================================================================

enum { kCwApprox = 0, kCwRow1D = 1, kCwRow1DAbsorb = 2 };

// keep(i,j) <=> at least K entries of row i precede (i,j) and (Algorithm 1 only) at least K entries of column j do:
// the rank form of the greedy sweep under the (magnitude, row-major index) order.
template <int SOLVER, int DT, int M, int FMT>
__global__ __launch_bounds__(kCwThreads, M == 32 ? 4 : 1) void cw_mask_kernel(const CwArgs args)
{
    constexpr int NB = 64 / M;
    __shared__ uint32_t T[NB][M][M + 1];
    const CwMat md = args.m[cw_find(args, blockIdx.x)];
    const uint32_t lane = threadIdx.x, blk = lane / M, j = lane % M;
    const uint32_t K = args.K;
    double total = 0.0;
    for (uint32_t t = blockIdx.x - md.wg0; t < md.n_tiles; t += md.n_wg) {
        const CwTile p = cw_tile<(M == 32 && SOLVER == kCwApprox) ? 4 : 1>(md, t);
        // M = 32: the raw column is not held across the sorts (32 registers that cost a wavefront of occupancy); the
        // dense output, when asked for, reads it again
        constexpr bool kHoldRaw = M < 32;
        uint32_t raw[M], key[M];
        cw_load_column<DT, M>(md, p, key);
#pragma unroll
        for (int i = 0; i < M; i++) {
            if constexpr (kHoldRaw)
                raw[i] = key[i];
            key[i] = cw_key<DT>(key[i]);
        }
        // rows: lane j of the block takes row j.  The magnitudes go to the transposition buffer first; the column pass
        // below is then their last use in registers
        __syncthreads();                                  // the previous tile's readers are done
#pragma unroll
        for (int i = 0; i < M; i++)
            T[blk][i][j] = key[i];
        uint32_t keep = seg_mask<M>();
        if constexpr (SOLVER == kCwApprox) {
            keep = ~cw_pruned<DT, M>(key, K) & seg_mask<M>();
        }
        __syncthreads();
        {
            uint32_t rk[M];
#pragma unroll
            for (int c = 0; c < M; c++)
                rk[c] = T[blk][j][c];
            // back to columns: bit c of row j's word becomes bit j of column c's
            keep &= cw_transpose<M>(~cw_pruned<DT, M>(rk, K) & seg_mask<M>());
        }
        if (md.mask)
            cw_store_mask<M, FMT>(md, p, keep);
        float acc = 0.f;
#pragma unroll
        for (int i = 0; i < M; i++) {
            // M = 32: the lane's magnitudes come back from the transposition buffer (its own writes), so that they hold
            // no registers while the rows are sorted
            const uint32_t mag = M == 32 ? T[blk][i][j] : key[i];
            acc += ((keep >> i) & 1u) ? __uint_as_float(mag) : 0.f;
        }
        total += (double)wave_sum(acc);
        if (md.aux) {
            // dense masked copy; with absorption the mean of a row group's pruned weights goes to its kept ones
            constexpr size_t ES = DT == kF32 ? 4 : 2;
            if constexpr (!kHoldRaw)
                cw_load_column<DT, M>(md, p, raw);        // every entry is read and written by the same lane: in place is fine
            char *orow = (char *)md.aux + ((size_t)p.br * M * md.ld_aux + p.col0) * ES;      // same in every lane
#pragma unroll
            for (int i = 0; i < M; i++) {
                const bool k = (keep >> i) & 1u;
                uint32_t o = k ? raw[i] : 0u;
                if constexpr (SOLVER == kCwRow1DAbsorb) {
                    const float v = DT == kF32 ? __uint_as_float(raw[i]) : __uint_as_float(raw[i] << 16);
                    const float ps = seg_sum<M>(k ? 0.f : v);
                    const uint32_t pc = (uint32_t)M - (uint32_t)__builtin_popcount(seg_of<M>(lm(k), blk));
                    const float mean = (pc != 0u && pc != (uint32_t)M) ? ps / (float)pc : 0.f;
                    const float res = k ? v + mean : 0.f;
                    o = DT == kF32 ? __float_as_uint(res) : f32_to_bf16_rne(res);
                }
                if (p.active) {
                    if constexpr (DT == kF32)
                        ((uint32_t *)orow)[threadIdx.x] = o;
                    else
                        ((uint16_t *)orow)[threadIdx.x] = (uint16_t)o;
                }
                orow += (size_t)md.ld_aux * ES;
            }
        }
    }
    if (args.partials && threadIdx.x == 0)
        ((double *)args.partials)[args.partial0 + blockIdx.x] = total;
}

// =====================================================================================================================
// Exact: the optimum of Eq. 3 per block by successive shortest augmenting paths on the network of Fig. 3.
//
// Costs are integers (|W| scaled by a power of two so that the block maximum lies in [2^(S-1), 2^S), truncated), so
// path sums are exact and label-correcting search terminates with a predecessor forest.  Start: every column prunes
// its K lightest rows (cheapest for the row counts it has).  While some row has more than K pruned entries: labels of
// all rows from the rows with excess (Bellman-Ford, alternating a column step -- reach column j through a pruned
// entry, lane j holds column j -- and a row step -- leave it through an unpruned entry, lane j holds row j; labels
// and predecessors are exchanged through LDS), then one augmentation per block along the predecessor chain of its
// first reachable row that lacks pruned entries.  At convergence every predecessor edge is tight, so the pruning stays
// cheapest for its row counts, and after (total excess) augmentations it is the optimum.
// =====================================================================================================================

constexpr int kCwInf = 0x70000000;        // unreachable; kCwInf - 2^S is still above kCwReachable
constexpr int kCwReachable = 0x40000000;  // |label| <= (M - 1) * 2^S < 2^30
constexpr uint32_t kCwNone = 0xFFu;

constexpr int cw_cost_bits(int M) { return M == 32 ? 25 : M == 16 ? 26 : 27; }

template <int DT, int M, int FMT>
__global__ __launch_bounds__(kCwThreads, M == 32 ? 3 : 1) void cw_exact_kernel(const CwArgs args)
{
    constexpr int NB = 64 / M;
    constexpr int S = cw_cost_bits(M);
    static_assert((M - 1) * (1ll << S) < kCwReachable, "labels must stay below the reachability threshold");
    __shared__ uint32_t T[NB][M][M + 1];
    __shared__ int DROW[NB][M], DCOL[NB][M];
    __shared__ uint32_t PROW[NB][M], PCOL[NB][M];
    __shared__ uint32_t PK[NB][M];
    const CwMat md = args.m[cw_find(args, blockIdx.x)];
    const uint32_t lane = threadIdx.x, blk = lane / M, j = lane % M;
    const uint32_t K = args.K;
    double total = 0.0;
    for (uint32_t t = blockIdx.x - md.wg0; t < md.n_tiles; t += md.n_wg) {
        const CwTile p = cw_tile(md, t);
        uint32_t key[M];
        cw_load_column<DT, M>(md, p, key);
#pragma unroll
        for (int i = 0; i < M; i++)
            key[i] = cw_key<DT>(key[i]);
        // ---- integer costs, by column (ccol) and, through LDS, by row (crow) ----
        uint32_t kmax = 0;
#pragma unroll
        for (int i = 0; i < M; i++)
            kmax = key[i] > kmax ? key[i] : kmax;
        kmax = seg_max<M>(kmax);
        const uint32_t emax = (kmax >> 23) ? (kmax >> 23) : 1u;
        int ccol[M], crow[M];
#pragma unroll
        for (int i = 0; i < M; i++) {
            const uint32_t e = key[i] >> 23;
            const uint32_t mant = (key[i] & 0x7FFFFFu) | (e ? 0x800000u : 0u);
            const uint32_t sh = emax - (e ? e : 1u);
            ccol[i] = sh < 32u ? (int)((mant << (S - 24)) >> sh) : 0;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < M; i++)
            T[blk][i][j] = (uint32_t)ccol[i];
        __syncthreads();
        uint32_t xcol = 0, xrow = 0;       // bit i of xcol: (i, j) pruned; bit c of xrow: (j, c) pruned
        {
            // ---- start under row prices: column j prunes the K rows with the smallest cost + price.  Whatever the
            // prices, that is the cheapest pruning for the row counts it has, which is all the searches below ask of
            // their start; the prices are moved against the imbalance (price_i += step * (count_i - K), the step
            // shrinking per round) and the round with the least excess is kept.  Lane j owns the price of row j; the
            // prices travel through LDS, the counts come from the transposed flag words.  Rounds, first step (as a
            // fraction of the largest cost) and decay: M = 32: 16, 1/64, 12/16 (more rounds leave fewer searches but
            // cost more than those, measured; excess left on random blocks 36 -> 0.5); M = 16: 20, 1/32, 12/16;
            // M <= 8: 12, 3/64, 11/16.  Keys: (cost + price) << log2 M | tie-break < 2^31.
            constexpr int ROUNDS = M == 32 ? 16 : M == 16 ? 20 : 12;
            constexpr int LOGM = M == 32 ? 5 : M == 16 ? 4 : M == 8 ? 3 : 2;
            static_assert(S + 1 + LOGM <= 31, "keys fit 31 bits");
            // cost << log2 M | tie-break, the tie-break of entry (i, j) being (i - j) mod M: columns with equal costs
            // (blocks of an unstructured-sparse matrix are full of zeros) then prune different rows, a band, instead of
            // all the same ones, which no row price could tell apart (4096^2 with 90 % zeros at 16:32: 3.3 -> 0.55 ms)
            uint32_t ckey[M];
#pragma unroll
            for (int i = 0; i < M; i++)
                ckey[i] = ((uint32_t)ccol[i] << LOGM) | (((uint32_t)i - j) & (uint32_t)(M - 1));
            int pr = 1 << (S - 1), best_pr = pr;
            uint32_t best = 0xFFFFFFFFu;
            int step = M == 32 ? (1 << (S - 6)) : M == 16 ? (4 << (S - 7)) : (3 << (S - 6));
            for (int round = 0; round <= ROUNDS + 1; round++) {
                const bool last = round == ROUNDS + 1;        // the kept prices once more, for their flags
                __syncthreads();
                PK[blk][j] = (uint32_t)(last ? best_pr : pr) << LOGM;
                __syncthreads();
                uint32_t k[M];
#pragma unroll
                for (int i = 0; i < M; i++)
                    k[i] = ckey[i] + PK[blk][i];
                const uint32_t t = cw_threshold<M>(k, K);
                uint32_t w = 0;
#pragma unroll
                for (int i = M - 1; i >= 0; i--)
                    lm_shift_in(w, lm(k[i] < t));
                const uint32_t wr = cw_transpose<M>(w);
                xcol = w;
                xrow = wr;
                if (last)
                    break;
                const uint32_t n = (uint32_t)__builtin_popcount(wr);
                uint32_t e = seg_sum_u32<M>(n > K ? n - K : 0u);
                e = p.active ? e : 0u;
                const bool better = e < best;
                best = better ? e : best;
                best_pr = better ? pr : best_pr;
                if (!__any(best != 0u))
                    break;                                   // every block balanced: this round's flags are the start
                const int q = pr + step * ((int)n - (int)K);
                pr = q < 1 ? 1 : q > (1 << S) - 1 ? (1 << S) - 1 : q;
                step = (step * (M <= 8 ? 11 : 12)) >> 4;
            }
            // the plain costs again, out of the keys (only one of the two arrays holds registers at a time)
#pragma unroll
            for (int i = 0; i < M; i++)
                ccol[i] = (int)(ckey[i] >> LOGM);
        }
#pragma unroll
        for (int c = 0; c < M; c++)
            crow[c] = (int)T[blk][j][c];
        // a block outside the matrix takes no part: it counts as balanced
        uint32_t cnt = p.active ? (uint32_t)__builtin_popcount(xrow) : K;

        // ---- augment until no row has more than K pruned entries; at most M*K augmentations per block ----
        for (int round = 0; round < M * M; round++) {
            const bool excess = cnt > K;
            const bool blk_excess = seg_of<M>(lm(excess), blk) != 0u;
            if (!__any(excess))
                break;
            int drow = excess ? 0 : kCwInf;
            uint32_t prow = kCwNone;
            __syncthreads();
            DROW[blk][j] = drow;
            PROW[blk][j] = prow;
            __syncthreads();
            // Labels only ever fall, and a predecessor changes only when its label falls strictly: with exact integer
            // sums and no negative cycle the predecessor graph is then a forest, also among entries of equal cost.
            int dcol = kCwInf;
            uint32_t pcol = 0;
            for (int it = 0; it <= M; it++) {
                // column step: the cheapest way into column j, through a pruned entry of a reached row
#pragma unroll
                for (int i = 0; i < M; i++) {
                    const int d = DROW[blk][i];
                    const int v = d - ccol[i];
                    const bool better = ((xcol >> i) & 1u) && d < kCwReachable && v < dcol;
                    dcol = better ? v : dcol;
                    pcol = better ? (uint32_t)i : pcol;
                }
                DCOL[blk][j] = dcol;
                PCOL[blk][j] = pcol;
                __syncthreads();
                // row step: leave a column through an unpruned entry of row j
                bool changed = false;
#pragma unroll
                for (int c = 0; c < M; c++) {
                    const int v = DCOL[blk][c] + crow[c];
                    const bool better = !((xrow >> c) & 1u) && v < drow;
                    drow = better ? v : drow;
                    prow = better ? (uint32_t)c : prow;
                    changed = changed || better;
                }
                DROW[blk][j] = drow;
                PROW[blk][j] = prow;
                __syncthreads();
                if (!__any(changed))
                    break;
            }
            // the block's first reachable row that lacks pruned entries takes its chain
            const uint32_t cand = seg_of<M>(lm(cnt < K && drow < kCwReachable), blk);
            bool walking = blk_excess && cand != 0u;
            if (!__any(walking))
                break;                      // cannot happen for 0 < K < M; guards against looping on corrupt state
            const uint32_t target = walking ? (uint32_t)__builtin_ctz(cand) : 0u;
            uint32_t r = target, src = kCwNone;
            for (int step = 0; step < M && __any(walking); step++) {
                if (walking) {
                    const uint32_t c = PROW[blk][r];
                    if (c == kCwNone) {
                        src = r;
                        walking = false;
                    } else {
                        const uint32_t f = PCOL[blk][c];          // (r, c) becomes pruned, (f, c) becomes unpruned
                        if (j == c)
                            xcol ^= (1u << r) | (1u << f);
                        if (j == r || j == f)
                            xrow ^= 1u << c;
                        r = f;
                    }
                }
            }
            if (walking) {                   // chain of full length: its last row must be the source
                src = (PROW[blk][r] == kCwNone) ? r : kCwNone;
            }
            if (src != kCwNone)
                cnt += (j == target ? 1u : 0u) - (j == src ? 1u : 0u);
        }
        const uint32_t keep = ~xcol & seg_mask<M>();
        cw_store_mask<M, FMT>(md, p, keep);
        if constexpr (M == 32) {
            // the magnitudes are read again for the objective: they hold no registers during the solve
            cw_load_column<DT, M>(md, p, key);
#pragma unroll
            for (int i = 0; i < M; i++)
                key[i] = cw_key<DT>(key[i]);
        }
        float acc = 0.f;
#pragma unroll
        for (int i = 0; i < M; i++)
            acc += (p.active && ((keep >> i) & 1u)) ? __uint_as_float(key[i]) : 0.f;
        total += (double)wave_sum(acc);
    }
    if (args.partials && threadIdx.x == 0)
        ((double *)args.partials)[args.partial0 + blockIdx.x] = total;
}

// =====================================================================================================================
// Score (Eq. 3's objective and constraints for a given mask)
// =====================================================================================================================

template <int DT, int M, int FMT>
__global__ __launch_bounds__(kCwThreads) void cw_score_kernel(const CwArgs args)
{
    const CwMat md = args.m[cw_find(args, blockIdx.x)];
    const uint32_t lane = threadIdx.x, blk = lane / M, j = lane % M;
    const uint32_t N = args.N;
    double retained = 0.0, total = 0.0;
    unsigned long long kept = 0, rowv = 0, colv = 0, rowne = 0, colne = 0;
    for (uint32_t t = blockIdx.x - md.wg0; t < md.n_tiles; t += md.n_wg) {
        const CwTile p = cw_tile<M == 32 ? 4 : 1>(md, t);
        const uint32_t bits = cw_load_mask<M, FMT>(md, p);
        uint32_t raw[M];
        cw_load_column<DT, M>(md, p, raw);
        float ret = 0.f, tot = 0.f;
#pragma unroll
        for (int i = 0; i < M; i++) {
            const float v = __uint_as_float(cw_key<DT>(raw[i]));
            tot += v;
            ret += ((bits >> i) & 1u) ? v : 0.f;
        }
        uint32_t rowcnt = 0;                       // kept entries of row j of the block
#pragma unroll
        for (int i = 0; i < M; i++) {
            const uint32_t rb = seg_of<M>(lm((bits >> i) & 1u), blk);
            rowcnt = (j == (uint32_t)i) ? (uint32_t)__builtin_popcount(rb) : rowcnt;
        }
        const uint32_t colcnt = (uint32_t)__builtin_popcount(bits);
        const uint32_t a = p.active ? 1u : 0u;
        const uint32_t w_kept = wave_sum(colcnt);
        const uint32_t w_flags = wave_sum((a & (rowcnt > N ? 1u : 0u)) | ((a & (colcnt > N ? 1u : 0u)) << 8) |
                                          ((a & (rowcnt != N ? 1u : 0u)) << 16) | ((a & (colcnt != N ? 1u : 0u)) << 24));
        kept += w_kept;
        rowv += w_flags & 0xFFu; colv += (w_flags >> 8) & 0xFFu; rowne += (w_flags >> 16) & 0xFFu; colne += w_flags >> 24;
        const float blk_ret = seg_sum<M>(ret);
        if (md.aux && p.active && j == 0u)
            ((float *)md.aux)[(size_t)p.br * (md.cols / M) + p.col / M] = blk_ret;
        retained += (double)wave_sum(ret);
        total += (double)wave_sum(tot);
    }
    if (threadIdx.x == 0) {
        ScorePartial *out = (ScorePartial *)args.partials + args.partial0 + blockIdx.x;
        out->retained = retained; out->total = total;
        out->kept = kept; out->rowv = rowv; out->colv = colv; out->rowne = rowne; out->colne = colne;
    }
}

// =====================================================================================================================
// Apply + pack, two passes in one launch: groups along rows (vals, idx), then groups down columns (valsT, idxT).
// A workgroup takes 32 lines x 8 consecutive groups (so the position bits it assembles are whole bytes, 8 * N * log2 M
// bits, wherever the line does not end): the weights and keep flags of that piece are loaded with neighbouring lanes on
// neighbouring addresses and staged in LDS, one thread per group then compacts its group in place (slot s never lies
// behind position s), and the compacted values leave as one contiguous run per line.  The LDS pitches are chosen per
// pass so that the threads of a wavefront (8 lines x 8 groups in the row pass, 32 lines x 2 groups in the column pass)
// fall into different banks.
// =====================================================================================================================

constexpr int kCwPackThreads = 256;

struct CwPack {
    const void *w;
    const void *mask;
    void *vals, *idx, *valsT, *idxT;
    uint32_t rows, cols, ld, mask_ld;
    uint32_t wg0, row_wgs;   // first workgroup of this matrix; how many of its workgroups do the row pass
};

struct CwPackArgs {
    CwPack d[kMaxCwBatch];
    uint32_t n, N;
};
static_assert(sizeof(CwPackArgs) <= 16384, "descriptor table is sized to stay a small kernel argument");

template <int M>
struct CwLog2 {
    static constexpr int v = (M == 4) ? 2 : (M == 8) ? 3 : (M == 16) ? 4 : 5;
};

// where a piece lies: matrix, pass and position (all the same in every thread of the workgroup)
struct CwPiece {
    const void *w;
    const unsigned char *mask;
    void *vals;              // vals / valsT of the pass
    unsigned char *idx;      // idx / idxT of the pass
    uint32_t ld, mask_ld;
    uint32_t n_lines, gpl;   // lines of the pass, groups per line
    uint32_t lb, ch;         // block of 32 lines, chunk of 8 groups
    uint32_t g_here;         // groups in this chunk (the last chunk of a line may be short)
    bool transposed;
};

template <int M>
__device__ __forceinline__ CwPiece cw_piece(const CwPackArgs &args, uint32_t piece)
{
    int lo = 0, hi = (int)args.n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (args.d[mid].wg0 <= piece)
            lo = mid;
        else
            hi = mid - 1;
    }
    const CwPack &d = args.d[lo];
    CwPiece p;
    uint32_t wg = piece - d.wg0;
    p.transposed = wg >= d.row_wgs;
    if (p.transposed)
        wg -= d.row_wgs;
    // the pass's view: n_lines lines of gpl groups; element q of group g of line L is W[L][g*M + q] (row pass) or
    // W[g*M + q][L] (column pass)
    p.w = d.w; p.mask = (const unsigned char *)d.mask; p.ld = d.ld; p.mask_ld = d.mask_ld;
    p.vals = p.transposed ? d.valsT : d.vals;
    p.idx = (unsigned char *)(p.transposed ? d.idxT : d.idx);
    p.n_lines = p.transposed ? d.cols : d.rows;
    p.gpl = (p.transposed ? d.rows : d.cols) / M;
    const uint32_t chunks = (p.gpl + 7u) / 8u;
    p.lb = wg / chunks;
    p.ch = wg - p.lb * chunks;
    p.g_here = min(8u, p.gpl - p.ch * 8u);
    return p;
}

// One piece, one pass (T: the column pass).  The pass is a template argument so that everything that depends on it --
// which thread loads what, where it lands in LDS -- is a constant per load instead of arithmetic per load.
template <int DT, int M, int FMT, bool T, int WORDS>
__device__ __forceinline__ void cw_pack_piece(const CwPiece &p, const uint32_t N, uint32_t *WT, uint32_t *KF,
                                              uint32_t (*IDX)[WORDS])
{
    constexpr int IB = CwLog2<M>::v;
    constexpr size_t ES = DT == kF32 ? 4 : 2;
    constexpr uint32_t GP = M + 1;                       // words per group in LDS (one of padding)
    constexpr uint32_t PITCH_ROW = ((8 * GP + 55) / 64) * 64 + 8;   // = 8 (mod 64), >= 8 * GP
    constexpr uint32_t pitch = T ? PITCH_ROW + 1 : PITCH_ROW;       // column pass: odd
    constexpr uint32_t KP = 8 * M + 4;                   // bytes of keep flags per line
    constexpr uint32_t EPL = 8u * M;                     // elements per line of a full piece
    constexpr uint32_t STEPS = 32u * EPL / kCwPackThreads;
    constexpr uint32_t DL = T ? 0u : kCwPackThreads / EPL;   // lines a thread moves down per load (row pass)
    constexpr uint32_t DE = T ? 8u : 0u;                      // elements it moves along the line (column pass)
    const uint32_t tid = threadIdx.x;
    unsigned char *kf = (unsigned char *)KF;
    const uint32_t e_here = p.g_here * M;

    // ---- loads.  All of a thread's loads are issued back to back (up to 32 of each kind), none inside a branch (its
    // result would be waited for at the join); entries outside the matrix read element (0, 0) and are dropped below.
    // row pass: neighbouring lanes = neighbouring elements of a line; column pass: neighbouring lines (columns).  From
    // one load of a thread to its next the matrix row advances by the same amount, DL + DE rows.
    const uint32_t l0 = T ? (tid & 31u) : (tid / EPL);
    const uint32_t e0 = T ? (tid >> 5) : (tid % EPL);
    const uint32_t line0 = p.lb * 32u + l0;
    const uint32_t lines_left = p.n_lines > line0 ? p.n_lines - line0 : 0u;
    const uint32_t elems_left = e_here > e0 ? e_here - e0 : 0u;
    // the first n_in of the thread's entries lie inside the matrix
    const uint32_t n_in = T ? (lines_left ? (elems_left + 7u) / 8u : 0u) : (elems_left ? (lines_left + DL - 1u) / DL : 0u);
    uint32_t v[STEPS], f[STEPS];
    {
        const uint32_t r0 = T ? p.ch * EPL + e0 : line0, c0 = T ? line0 : p.ch * EPL + e0;
        const char *wp = (const char *)p.w + ((size_t)r0 * p.ld + c0) * ES;
        const unsigned char *mp = p.mask + (size_t)r0 * p.mask_ld + (FMT == kMaskU8 ? c0 : (c0 >> 3));
        const size_t wstep = (size_t)__builtin_amdgcn_readfirstlane((DL + DE) * (uint32_t)ES) * __builtin_amdgcn_readfirstlane(p.ld);
        const size_t mstep = (size_t)(DL + DE) * __builtin_amdgcn_readfirstlane(p.mask_ld);
#pragma unroll
        for (uint32_t b = 0; b < STEPS; b++) {
            const bool in = b < n_in;
            const char *wa = in ? wp : (const char *)p.w;
            const unsigned char *ma = in ? mp : p.mask;
            if constexpr (DT == kF32)
                v[b] = __builtin_nontemporal_load((const uint32_t *)wa);
            else
                v[b] = (uint32_t)__builtin_nontemporal_load((const uint16_t *)wa);
            if constexpr (FMT == kMaskU8)
                f[b] = (uint32_t)*ma;
            else
                f[b] = ((uint32_t)*ma >> (c0 & 7u)) & 1u;
            wp += wstep;
            mp += mstep;
        }
    }
    for (uint32_t k = tid; k < 32u * WORDS; k += kCwPackThreads)
        (&IDX[0][0])[k] = 0;
    // ---- stage the piece: weights as words, keep flags as bytes (0 / 1); the place of load b is the place of load 0
    // plus a constant ----
    {
        uint32_t *w0 = WT + l0 * pitch + (e0 / M) * GP + (e0 % M);
        unsigned char *k0 = kf + l0 * KP + e0;
#pragma unroll
        for (uint32_t b = 0; b < STEPS; b++) {
            // row pass: DL lines further down; column pass: 8 elements further along (e0 < 8, so e0 % M + 8 * b stays
            // inside the group for 8 * (b % (M / 8)) and moves on by whole groups otherwise)
            const uint32_t woff = T ? ((8u * b) / M) * GP + (8u * b) % M : b * DL * pitch;
            const uint32_t koff = T ? 8u * b : b * DL * KP;
            if (b < n_in) {
                w0[woff] = v[b];
                k0[koff] = (unsigned char)(f[b] != 0u ? 1u : 0u);
            }
        }
    }
    __syncthreads();
    // ---- one thread per group: slots, compaction in place, position codes ----
    // row pass: eight neighbouring threads take eight neighbouring groups of a line; column pass: 32 neighbouring
    // threads take 32 neighbouring lines
    const uint32_t ll = T ? (tid & 31u) : (tid >> 3);
    const uint32_t gl = T ? (tid >> 5) : (tid & 7u);
    if (p.lb * 32u + ll < p.n_lines && gl < p.g_here) {
        uint32_t kb = 0;
#pragma unroll
        for (int q4 = 0; q4 < M / 4; q4++) {
            const uint32_t f4 = KF[(ll * KP + gl * M) / 4 + q4];          // four flag bytes, each 0 or 1
            kb |= ((f4 * 0x01020408u) >> 24) << (4 * q4);
        }
        // slots: the kept positions in order (the first N if the mask keeps more), then the lowest other positions
        uint32_t sel = kb, cnt = (uint32_t)__builtin_popcount(kb);
        while (cnt > N) {
            sel &= ~(0x80000000u >> __builtin_clz(sel));
            cnt--;
        }
        uint32_t z = ~sel & seg_mask<M>(), chosen = sel;
        for (uint32_t need = N - cnt; need > 0; need--) {
            const uint32_t low = z & (0u - z);
            chosen |= low;
            z ^= low;
        }
        uint32_t *grp = &WT[ll * pitch + gl * GP];
        uint32_t gv[M];
#pragma unroll
        for (int q = 0; q < M; q++)
            gv[q] = grp[q];
        uint32_t sl = 0, off = gl * N * IB;
#pragma unroll
        for (int q = 0; q < M; q++) {
            if ((chosen >> q) & 1u) {
                grp[sl] = ((sel >> q) & 1u) ? gv[q] : 0u;                  // the group is compacted in place
                const unsigned long long code = (unsigned long long)q << (off & 31u);
                atomicOr(&IDX[ll][off >> 5], (uint32_t)code);
                if ((uint32_t)(code >> 32))
                    atomicOr(&IDX[ll][(off >> 5) + 1], (uint32_t)(code >> 32));
                sl++;
                off += IB;
            }
        }
    }
    __syncthreads();
    // ---- copy-out: per line one run of g_here * N values and one of position bytes.  A thread keeps its place x in
    // the run from line to line, so which group and slot that is is worked out once ----
    const size_t vpitch = (size_t)p.gpl * N;
    const uint32_t run = p.g_here * N;
    const float inv_n = 1.0f / (float)N;
    constexpr uint32_t XS = (8u * (M - 1) + 63u) / 64u;          // places per thread: a run has at most 8 * (M - 1) values
    uint32_t src[XS];
#pragma unroll
    for (uint32_t k = 0; k < XS; k++) {
        const uint32_t x = (tid & 63u) + 64u * k;
        const uint32_t g = (uint32_t)(((float)x + 0.5f) * inv_n);     // x / N, exact for x < 256, N < 32
        src[k] = g * GP + (x - g * N);
    }
    const uint32_t first_line = tid >> 6;
    if (p.lb * 32u + first_line < p.n_lines) {
        char *out = (char *)p.vals + ((size_t)(p.lb * 32u + first_line) * vpitch + (size_t)p.ch * 8u * N + (tid & 63u)) * ES;
        const size_t out_step = (size_t)__builtin_amdgcn_readfirstlane((uint32_t)(kCwPackThreads / 64)) * vpitch * ES;
        const uint32_t n_lines_here = min(32u, p.n_lines - p.lb * 32u);
        for (uint32_t l = first_line; l < n_lines_here; l += kCwPackThreads / 64) {
#pragma unroll
            for (uint32_t k = 0; k < XS; k++) {
                if ((tid & 63u) + 64u * k < run) {
                    const uint32_t val = WT[l * pitch + src[k]];
                    if constexpr (DT == kF32)
                        *(uint32_t *)(out + 64u * k * ES) = val;
                    else
                        *(uint16_t *)(out + 64u * k * ES) = (uint16_t)val;
                }
            }
            out += out_step;
        }
    }
    // the chunk's position bits start on a byte boundary of the line: 8 groups * N * IB bits = N * IB bytes
    const size_t pitch_b = ((size_t)p.gpl * N * IB + 7) / 8;
    const uint32_t nbytes = (p.g_here * N * IB + 7u) / 8u;
    for (uint32_t k = tid; k < 32u * nbytes; k += kCwPackThreads) {
        const uint32_t l2 = k / nbytes, x = k - l2 * nbytes;
        if (p.lb * 32u + l2 < p.n_lines)
            p.idx[(size_t)(p.lb * 32u + l2) * pitch_b + (size_t)p.ch * N * IB + x] = ((const unsigned char *)&IDX[l2][0])[x];
    }
}

// One workgroup per piece.  (Persistent workgroups that load their next piece into registers while they compact the
// current one were slower, 322 against 262 us on 8192^2 fp32 16:32: all workgroups then load at the same moments.)
template <int DT, int M, int FMT>
__global__ __launch_bounds__(kCwPackThreads) void cw_pack_kernel(const CwPackArgs args)
{
    constexpr int IB = CwLog2<M>::v;
    constexpr int WORDS = (8 * (M - 1) * IB + 31) / 32 + 2;
    constexpr uint32_t GP = M + 1;
    constexpr uint32_t PITCH_ROW = ((8 * GP + 55) / 64) * 64 + 8;
    constexpr uint32_t KP = 8 * M + 4;
    __shared__ uint32_t WT[32 * (PITCH_ROW + 1)];
    __shared__ uint32_t KF[32 * KP / 4];
    __shared__ uint32_t IDX[32][WORDS];
    const CwPiece p = cw_piece<M>(args, blockIdx.x);
    if (p.transposed)
        cw_pack_piece<DT, M, FMT, true, WORDS>(p, args.N, WT, KF, IDX);
    else
        cw_pack_piece<DT, M, FMT, false, WORDS>(p, args.N, WT, KF, IDX);
}

// =====================================================================================================================
// Host side
// =====================================================================================================================

static void cw_magic_div(uint32_t d, uint32_t *mul, uint32_t *shift)
{
    uint32_t l = 0;
    while ((1ull << l) < d)
        l++;
    const uint32_t k = 31 + l;
    *mul = (uint32_t)(((1ull << k) / d) + 1);
    *shift = k;
}

// workgroups a matrix gets: one per tile at M = 32; for M <= 16 (the slow path of an unaligned matrix) never more than
// the per-workgroup partial results the documented workspace bound provides for (one per 256 strips of M rows x 4
// columns), each workgroup striding over several tiles
static uint32_t cw_wgs(int64_t rows, int64_t cols, int M, uint32_t n_tiles)
{
    if (M == 32)
        return n_tiles;
    const uint64_t strips = (uint64_t)((rows + M - 1) / M) * (uint64_t)((cols + 3) / 4);
    const uint64_t cap = (strips + kThreads - 1) / kThreads;
    return (uint32_t)(n_tiles < cap ? n_tiles : cap);
}

size_t cw_workgroups(int64_t rows, int64_t cols, int M)
{
    return cw_wgs(rows, cols, M, (uint32_t)((cols + 63) / 64) * (uint32_t)(rows / M));
}

static void cw_fill(CwMat &m, const void *w, int64_t rows, int64_t cols, int64_t ld, void *mask, int64_t mask_ld, int M,
                    uint32_t wg0)
{
    m.w = w; m.mask = mask; m.aux = nullptr;
    m.ld = (uint32_t)ld; m.mask_ld = (uint32_t)mask_ld; m.ld_aux = 0; m.cols = (uint32_t)cols;
    m.tpr = (uint32_t)((cols + 63) / 64);
    m.n_tiles = m.tpr * (uint32_t)(rows / M);
    m.wg0 = wg0;
    m.n_wg = cw_wgs(rows, cols, M, m.n_tiles);
    cw_magic_div(m.tpr, &m.div_mul, &m.div_shift);
}

typedef void (*cw_kernel_t)(const CwArgs);

#define CW_PICK_M(KERN, ...)                                                                                         \
    (M == 4 ? KERN<__VA_ARGS__, 4, kMaskU8> : M == 8 ? KERN<__VA_ARGS__, 8, kMaskU8>                                 \
     : M == 16 ? KERN<__VA_ARGS__, 16, kMaskU8> : KERN<__VA_ARGS__, 32, kMaskU8>)
#define CW_PICK_M_BITS(KERN, ...)                                                                                    \
    (M == 4 ? KERN<__VA_ARGS__, 4, kMaskBits> : M == 8 ? KERN<__VA_ARGS__, 8, kMaskBits>                             \
     : M == 16 ? KERN<__VA_ARGS__, 16, kMaskBits> : KERN<__VA_ARGS__, 32, kMaskBits>)

static cw_kernel_t cw_pick_mask(int solver, int dt, int M, int mf)
{
#define CW_ONE(SV)                                                                                                   \
    if (solver == SV)                                                                                                \
        return dt == kF32 ? (mf == kMaskU8 ? CW_PICK_M(cw_mask_kernel, SV, kF32) : CW_PICK_M_BITS(cw_mask_kernel, SV, kF32)) \
                          : (mf == kMaskU8 ? CW_PICK_M(cw_mask_kernel, SV, kBF16) : CW_PICK_M_BITS(cw_mask_kernel, SV, kBF16));
    CW_ONE(kCwApprox) CW_ONE(kCwRow1D) CW_ONE(kCwRow1DAbsorb)
#undef CW_ONE
    return nullptr;
}

// solver: 0 = Algorithm 1, 1 = exact, 2 = row pruning.  Arguments are validated by the caller; `ws` (if any objective
// is wanted) holds at least one double per workgroup.
int cw_run_mask(int solver, const tmask_mat *mats, int n_mats, int dt, int N, int M, int mf, void *ws, hipStream_t stream)
{
    bool want_obj = false;
    for (int i = 0; i < n_mats; i++)
        want_obj = want_obj || mats[i].objective;
    cw_kernel_t kern;
    if (solver == 1)
        kern = dt == kF32 ? (mf == kMaskU8 ? CW_PICK_M(cw_exact_kernel, kF32) : CW_PICK_M_BITS(cw_exact_kernel, kF32))
                          : (mf == kMaskU8 ? CW_PICK_M(cw_exact_kernel, kBF16) : CW_PICK_M_BITS(cw_exact_kernel, kBF16));
    else
        kern = cw_pick_mask(solver == 0 ? kCwApprox : kCwRow1D, dt, M, mf);
    uint32_t partial0 = 0;
    for (int first = 0; first < n_mats; first += kMaxCwBatch) {
        const int nb = n_mats - first < kMaxCwBatch ? n_mats - first : kMaxCwBatch;
        CwArgs args;
        memset(&args, 0, sizeof args);
        double *objective[kMaxCwBatch];
        uint32_t wg0[kMaxCwBatch + 1];
        uint32_t wgs = 0;
        for (int k = 0; k < nb; k++) {
            const tmask_mat &t = mats[first + k];
            cw_fill(args.m[k], t.w, t.rows, t.cols, t.ld, t.mask, t.mask_ld, M, wgs);
            objective[k] = t.objective;
            wg0[k] = wgs;
            wgs += args.m[k].n_wg;
        }
        wg0[nb] = wgs;
        args.n = (uint32_t)nb; args.K = (uint32_t)(M - N); args.N = (uint32_t)N;
        args.partial0 = partial0; args.partials = want_obj ? ws : nullptr;
        {
            ProfileScope prof(stream, first + kMaxCwBatch >= n_mats);
            hipLaunchKernelGGL(kern, dim3(wgs), dim3(kCwThreads), 0, stream, args);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return hip_fail(e, "column-wise mask kernel launch");
        if (want_obj) {
            const int rc = launch_objective_reduce(objective, wg0, nb, partial0, ws, stream);
            if (rc)
                return rc;
        }
        partial0 += wgs;
    }
    return TMASK_OK;
}

int cw_run_score(const tmask_mat *mats, int n_mats, int dt, int N, int M, int mf, tmask_score_out *out, float *per_block_obj,
                 void *ws, hipStream_t stream)
{
    const cw_kernel_t kern =
        dt == kF32 ? (mf == kMaskU8 ? CW_PICK_M(cw_score_kernel, kF32) : CW_PICK_M_BITS(cw_score_kernel, kF32))
                   : (mf == kMaskU8 ? CW_PICK_M(cw_score_kernel, kBF16) : CW_PICK_M_BITS(cw_score_kernel, kBF16));
    uint32_t partial0 = 0;
    size_t block0 = 0;
    for (int first = 0; first < n_mats; first += kMaxCwBatch) {
        const int nb = n_mats - first < kMaxCwBatch ? n_mats - first : kMaxCwBatch;
        CwArgs args;
        memset(&args, 0, sizeof args);
        uint32_t wg0[kMaxCwBatch + 1];
        uint32_t wgs = 0;
        for (int k = 0; k < nb; k++) {
            const tmask_mat &t = mats[first + k];
            cw_fill(args.m[k], t.w, t.rows, t.cols, t.ld, t.mask, t.mask_ld, M, wgs);
            args.m[k].aux = per_block_obj ? (void *)(per_block_obj + block0) : nullptr;
            block0 += (size_t)(t.rows / M) * (size_t)(t.cols / M);
            wg0[k] = wgs;
            wgs += args.m[k].n_wg;
        }
        wg0[nb] = wgs;
        args.n = (uint32_t)nb; args.K = (uint32_t)(M - N); args.N = (uint32_t)N;
        args.partial0 = partial0; args.partials = ws;
        {
            ProfileScope prof(stream, first + kMaxCwBatch >= n_mats);
            hipLaunchKernelGGL(kern, dim3(wgs), dim3(kCwThreads), 0, stream, args);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return hip_fail(e, "column-wise score kernel launch");
        const int rc = launch_score_reduce(wg0, nb, partial0, ws, out + first, stream);
        if (rc)
            return rc;
        partial0 += wgs;
    }
    return TMASK_OK;
}

// mode: 0 = Algorithm 1, 1 = row pruning, 2 = row pruning with mean absorption; out <- W (.) S, mask on request
int cw_run_dense(const tmask_mask_dense_desc *descs, int n, int dt, int N, int M, int mf, int mode, hipStream_t stream)
{
    const cw_kernel_t kern = cw_pick_mask(mode == 0 ? kCwApprox : mode == 1 ? kCwRow1D : kCwRow1DAbsorb, dt, M, mf);
    for (int first = 0; first < n; first += kMaxCwBatch) {
        const int nb = n - first < kMaxCwBatch ? n - first : kMaxCwBatch;
        CwArgs args;
        memset(&args, 0, sizeof args);
        uint32_t wgs = 0;
        for (int k = 0; k < nb; k++) {
            const tmask_mask_dense_desc &p = descs[first + k];
            cw_fill(args.m[k], p.w, p.rows, p.cols, p.ld, p.mask, p.mask_ld, M, wgs);
            args.m[k].aux = p.out;
            args.m[k].ld_aux = (uint32_t)p.ld_out;
            wgs += args.m[k].n_wg;
        }
        args.n = (uint32_t)nb; args.K = (uint32_t)(M - N); args.N = (uint32_t)N;
        {
            ProfileScope prof(stream, first + kMaxCwBatch >= n);
            hipLaunchKernelGGL(kern, dim3(wgs), dim3(kCwThreads), 0, stream, args);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return hip_fail(e, "column-wise mask + dense copy kernel launch");
    }
    return TMASK_OK;
}

typedef void (*cw_pack_kernel_t)(const CwPackArgs);

int cw_run_pack(const tmask_pack_desc *descs, int n, int dt, int N, int M, int mf, hipStream_t stream)
{
    const cw_pack_kernel_t kern =
        dt == kF32 ? (mf == kMaskU8 ? CW_PICK_M(cw_pack_kernel, kF32) : CW_PICK_M_BITS(cw_pack_kernel, kF32))
                   : (mf == kMaskU8 ? CW_PICK_M(cw_pack_kernel, kBF16) : CW_PICK_M_BITS(cw_pack_kernel, kBF16));
    for (int first = 0; first < n; first += kMaxCwBatch) {
        const int nb = n - first < kMaxCwBatch ? n - first : kMaxCwBatch;
        CwPackArgs args;
        memset(&args, 0, sizeof args);
        uint32_t wgs = 0;
        for (int k = 0; k < nb; k++) {
            const tmask_pack_desc &p = descs[first + k];
            CwPack &d = args.d[k];
            d.w = p.w; d.mask = p.mask; d.vals = p.vals; d.idx = p.idx; d.valsT = p.valsT; d.idxT = p.idxT;
            d.rows = (uint32_t)p.rows; d.cols = (uint32_t)p.cols; d.ld = (uint32_t)p.ld; d.mask_ld = (uint32_t)p.mask_ld;
            d.wg0 = wgs;
            d.row_wgs = (uint32_t)((p.rows + 31) / 32) * (uint32_t)((p.cols / M + 7) / 8);
            wgs += d.row_wgs + (uint32_t)((p.cols + 31) / 32) * (uint32_t)((p.rows / M + 7) / 8);
        }
        args.n = (uint32_t)nb; args.N = (uint32_t)N;
        {
            ProfileScope prof(stream, first + kMaxCwBatch >= n);
            hipLaunchKernelGGL(kern, dim3(wgs), dim3(kCwPackThreads), 0, stream, args);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return hip_fail(e, "column-wise pack kernel launch");
    }
    return TMASK_OK;
}

}  // namespace tmask

// tmask_exact for N = M/2, M = 8 or 16: the augmenting-path solver of tmask_solvers.hpp behind a
// load-balancing stage.
//
// The solver needs one augmentation per unit of row excess left by its start (every column prunes its
// K lightest rows), and lanes of a wavefront run in lockstep: a wavefront takes as long as its worst
// block while the others idle (measured: about 40 % of the lanes active).  The start's excess is cheap
// to predict, so each workgroup first sorts its blocks by predicted excess (stable counting sort,
// deterministic), exchanges the raw rows through LDS, and every wavefront then solves blocks that need
// about the same number of augmentations.  Results go back to each block's own place.
#pragma once
#include "tmask_device.hpp"
#include "tmask_networks.hpp"
#include "tmask_solvers.hpp"

namespace tmask {

template <int DT>
__device__ __forceinline__ void unpack_row(const u32x4 &r, uint32_t (&a)[16 / ((DT == kF32) ? 4 : 2)])
{
    const uint32_t d[4] = {r.x, r.y, r.z, r.w};
    if constexpr (DT == kF32) {
#pragma unroll
        for (int c = 0; c < 4; c++)
            a[c] = d[c] & 0x7FFFFFFFu;
    } else {
#pragma unroll
        for (int c = 0; c < 4; c++) {
            a[2 * c] = (d[c] << 16) & 0x7FFF0000u;
            a[2 * c + 1] = d[c] & 0x7FFF0000u;
        }
    }
}

// Row excess of the "every column prunes its K = M/2 lightest rows" start, predicted on the magnitude
// keys (low four bits replaced by the row index to break ties).  Same value in all lanes of a block.
template <int M, int C, int G>
__device__ __forceinline__ uint32_t predicted_excess(const uint32_t (&a)[M][C])
{
    constexpr int H = M / 2;
    uint32_t cnt[M];
#pragma unroll
    for (int i = 0; i < M; i++)
        cnt[i] = 0;
#pragma unroll
    for (int c = 0; c < C; c++) {
        uint32_t lo[H], hi[H];
#pragma unroll
        for (int i = 0; i < H; i++) {
            lo[i] = (a[i][c] & ~0xFu) | (uint32_t)i;
            hi[i] = (a[H + i][c] & ~0xFu) | (uint32_t)(H + i);
        }
        const uint32_t t = upper_half_min<H>(lo, hi);
#pragma unroll
        for (int i = 0; i < M; i++)
            cnt[i] += (((a[i][c] & ~0xFu) | (uint32_t)i) < t) ? 1u : 0u;
    }
    uint32_t e = 0;
#pragma unroll
    for (int i = 0; i < M; i++) {
        uint32_t n = cnt[i];
        if constexpr (G >= 2)
            n += quad_xor<1>(n);
        if constexpr (G == 4)
            n += quad_xor<2>(n);
        e += n > (uint32_t)H ? n - (uint32_t)H : 0u;
    }
    return e;
}

template <int DT, int M, int FMT>
__global__ __launch_bounds__(kThreads, (M == 8 ? 4 : 2)) void exact_balanced_kernel(const BatchArgs args)
{
    using Ge = Geo<DT, M>;
    constexpr int C = Ge::C, G = Ge::G;
    constexpr int NB = kThreads / G;          // blocks per workgroup
    constexpr int NBUCKET = 16;
    constexpr int RPR = M;                    // all rows of the block stay in LDS (M x 16 B x 256 lanes)
    __shared__ __attribute__((aligned(16))) u32x4 xraw[kThreads][RPR];
    __shared__ uint32_t sorig[NB];
    __shared__ uint32_t wcnt[kThreads / 64][NBUCKET];
    __shared__ double red[kThreads / 64];

    const uint32_t tile = blockIdx.x;
    const MatDev md = args.m[find_matrix(args, tile)];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t s = (tile - md.tile0) * kThreads + tid;
    const uint32_t gpos = tid & (G - 1);
    const bool valid = s < md.n_strips;

    // ---- load the block this lane sits on ----
    // Lanes past the matrix' last strip take part in the exchange with a filler block whose start has
    // no excess (a band of ones: entry (i, j) is 1 iff (i + j) mod M < M/2), so they cost the solver nothing.
    u32x4 raw[M];
#pragma unroll
    for (int i = 0; i < M; i++) {
        uint32_t d[4];
#pragma unroll
        for (int q = 0; q < 4; q++) {
            if constexpr (DT == kF32) {
                const uint32_t j = gpos * 4u + (uint32_t)q;
                d[q] = (((uint32_t)i + j) & (M - 1)) < (uint32_t)(M / 2) ? 0x3F800000u : 0u;
            } else {
                const uint32_t j = gpos * 8u + 2u * (uint32_t)q;
                d[q] = ((((uint32_t)i + j) & (M - 1)) < (uint32_t)(M / 2) ? 0x3F80u : 0u) |
                       ((((uint32_t)i + j + 1u) & (M - 1)) < (uint32_t)(M / 2) ? 0x3F800000u : 0u);
            }
        }
        raw[i] = u32x4{d[0], d[1], d[2], d[3]};
    }
    if (valid) {
        const StripPos pos = strip_pos(md, s);
        const char *base = (const char *)md.w + ((size_t)pos.br * M * md.ld + (size_t)pos.sc * C) * Ge::ES;
        const size_t row_bytes = (size_t)md.ld * Ge::ES;
#pragma unroll
        for (int i = 0; i < M; i++)
            raw[i] = __builtin_nontemporal_load((const u32x4 *)(base + i * row_bytes));
    }

    // ---- predicted work, stable counting sort of the workgroup's blocks by it ----
    uint32_t e;
    {
        uint32_t a[M][C];
#pragma unroll
        for (int i = 0; i < M; i++)
            unpack_row<DT>(raw[i], a[i]);
        e = predicted_excess<M, C, G>(a);
        e = e < (uint32_t)(NBUCKET - 1) ? e : (uint32_t)(NBUCKET - 1);
    }
    __builtin_amdgcn_sched_barrier(0);
    const bool leader = gpos == 0;
    uint32_t within = 0;
#pragma unroll
    for (int v = 0; v < NBUCKET; v++) {
        const lanemask_t m = lm(leader && e == (uint32_t)v);
        if (lane == 0)
            wcnt[wave][v] = (uint32_t)__builtin_popcountll(m);
        if (e == (uint32_t)v)
            within = (uint32_t)__builtin_popcountll(m & ((1ull << lane) - 1ull));
    }
    __syncthreads();
    uint32_t rank = within;
    for (int v = 0; v < NBUCKET; v++)
        for (int w = 0; w < (int)(kThreads / 64); w++)
            if ((uint32_t)v < e || ((uint32_t)v == e && (uint32_t)w < wave))
                rank += wcnt[w][v];
    // every lane of a block computed the same e; `within` and `rank` are meaningful in the leader only
    if constexpr (G == 2)
        rank = dpp_read<0xA0>(rank);   // quad_perm [0,0,2,2]
    if constexpr (G == 4)
        rank = dpp_read<0x00>(rank);   // quad_perm [0,0,0,0]
    const uint32_t slot = rank * G + gpos;
    if (leader)
        sorig[rank] = valid ? s : 0xFFFFFFFFu;

    // ---- exchange the raw rows: this lane continues with the block sorted into its position ----
#pragma unroll
    for (int round = 0; round < M / RPR; round++) {
        if (round)
            __syncthreads();
#pragma unroll
        for (int i = 0; i < RPR; i++)
            xraw[slot][i] = raw[round * RPR + i];
        __syncthreads();
#pragma unroll
        for (int i = 0; i < RPR; i++)
            raw[round * RPR + i] = xraw[tid][i];
    }
    const uint32_t my_s = sorig[tid / G];
    const bool my_valid = my_s != 0xFFFFFFFFu;

    // ---- solve ----
    __builtin_amdgcn_sched_barrier(0);
    float acc = 0.f;
    {
        uint32_t a[M][C], xcol[C], bits[M];
#pragma unroll
        for (int i = 0; i < M; i++) {
            unpack_row<DT>(raw[i], a[i]);
            // the raw rows end here: the keys must not be re-derived from them later
#pragma unroll
            for (int c = 0; c < C; c++)
                asm volatile("" : "+v"(a[i][c]));
        }
        exact_general<M, C, G>(a, (uint32_t)(M / 2), gpos, xcol);
#pragma unroll
        for (int i = 0; i < M; i++) {
            bits[i] = 0;
#pragma unroll
            for (int c = 0; c < C; c++)
                bits[i] |= (((xcol[c] >> i) & 1u) ^ 1u) << c;
        }
        if (my_valid) {
            const StripPos pos = strip_pos(md, my_s + gpos);
            store_mask<DT, M, FMT>(md, pos, bits);
            // the magnitudes are read again from LDS: they need not occupy registers during the solve
#pragma unroll
            for (int i = 0; i < M; i++) {
                uint32_t ar[C];
                unpack_row<DT>(xraw[tid][i], ar);
#pragma unroll
                for (int c = 0; c < C; c++)
                    acc += ((bits[i] >> c) & 1u) ? __uint_as_float(ar[c]) : 0.f;
            }
        }
    }
    if (args.partials) {
        const double t = block_sum_f32(acc, red);
        if (threadIdx.x == 0)
            ((double *)args.partials)[args.partial0 + tile] = t;
    }
}

}  // namespace tmask

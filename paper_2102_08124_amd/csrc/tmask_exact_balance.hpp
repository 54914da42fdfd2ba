// tmask_exact for N = M/2, M = 8 or 16: the augmenting-path solver of tmask_solvers.hpp behind a
// load-balancing stage.
//
// The solver needs one augmentation per unit of row excess left by its start, and lanes of a wavefront
// run in lockstep: a wavefront takes as long as its worst block while the others idle (measured: about
// 40 % of the lanes active).  So every lane first computes the start of the block it loaded (the price
// rounds included: uniform work, every lane busy), each workgroup sorts its blocks by the excess that is
// left (stable counting sort, deterministic), exchanges the raw rows and the start through LDS, and every
// wavefront then runs the searches of blocks that need about the same number of augmentations.  Results
// go back to each block's own place.
#pragma once
#include "tmask_device.hpp"
#include "tmask_networks.hpp"
#include "tmask_solvers.hpp"

namespace tmask {

// Magnitude keys (fp32 bit patterns) of the C values a lane holds of one row: four dwords (fp32, or eight bf16),
// or two dwords (four bf16) where a lane takes half a 16-byte strip.
template <int DT, int C>
__device__ __forceinline__ void unpack_row(const u32x4 &r, uint32_t (&a)[C])
{
    const uint32_t d[4] = {r.x, r.y, r.z, r.w};
    if constexpr (DT == kF32) {
        static_assert(C == 4, "an fp32 lane holds four columns");
#pragma unroll
        for (int c = 0; c < 4; c++)
            a[c] = d[c] & 0x7FFFFFFFu;
    } else {
#pragma unroll
        for (int c = 0; c < C / 2; c++) {
            a[2 * c] = (d[c] << 16) & 0x7FFF0000u;
            a[2 * c + 1] = d[c] & 0x7FFF0000u;
        }
    }
}

// Workgroups per compute unit: four at M = 8.  A bf16 lane holds eight columns of its block (an fp32 lane four) and
// would like 154 registers; held to 128 it keeps 35 values in scratch memory and is still 1-4 % faster than with
// three workgroups (headline set at 4:8: 1084 -> 1045 us).  At M = 16 eight columns of sixteen
// rows do not fit a lane at all (256 registers, spills): there a bf16 lane takes half a strip, four columns, and
// four lanes share a block as at fp32 (exact_half_strips; the host launches twice the workgroups).
// Where the raw rows wait for the lane that runs their block's searches: in LDS (M x 16 bytes per lane), except at
// M = 16, where those 64 KiB would hold the compute unit to two workgroups; there the rows are read from memory
// again (the second and third reading mostly hit the cache) and three workgroups fit, registers permitting
// (8192 x 8192 fp32: 890 -> 714 us; the M = 8 cases measured the same or 2-4 % slower without the LDS copy).
constexpr bool exact_half_strips(int dt, int M) { return dt == kBF16 && M == 16; }
constexpr bool exact_rows_in_lds(int dt, int M) { return M != 16; }
constexpr int exact_workgroups_per_cu(int dt, int M) { return M == 16 ? 3 : 4; }

// GENERAL: any N (K = args.K pruned per line); otherwise N = M/2.
template <int DT, int M, int FMT, bool GENERAL = false>
__global__ __launch_bounds__(kThreads, exact_workgroups_per_cu(DT, M)) void exact_balanced_kernel(const BatchArgs args)
{
    const uint32_t K = GENERAL ? args.K : (uint32_t)(M / 2);
    const uint32_t NKEEP = (uint32_t)M - K;
    constexpr bool PARK = exact_rows_in_lds(DT, M);
    using Ge = Geo<DT, M>;
    constexpr bool HALF = exact_half_strips(DT, M);
    constexpr int C = HALF ? 4 : Ge::C, G = HALF ? 4 : Ge::G;     // columns per lane, lanes per block
    constexpr int NB = kThreads / G;          // blocks per workgroup
    constexpr int NBUCKET = 16;
    static_assert(kThreads <= 256 && NBUCKET <= 16, "a lane number and an excess bucket share sixteen bits (ssrc)");
    constexpr int XPW = 32 / M;               // pruned-row sets (M bits per column) per exchanged word
    constexpr int XW = C / XPW;
    // PARK: the raw rows of every block stay in LDS, at the loading lane's place; else they are read from memory again
    __shared__ __attribute__((aligned(16))) u32x4 xraw[PARK ? kThreads : 1][M];
    __shared__ uint32_t xstart[kThreads][XW];
    __shared__ uint16_t ssrc[kThreads];
    __shared__ uint32_t sorig[NB];
    __shared__ uint32_t wcnt[kThreads / 64][NBUCKET];
    __shared__ double red[kThreads / 64];

    const uint32_t tile = blockIdx.x;
    const MatDev md = args.m[find_matrix(args, tile)];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t s = (tile - md.tile0) * kThreads + tid;
    const uint32_t gpos = tid & (G - 1);
    const bool valid = s < md.n_strips * (HALF ? 2u : 1u);      // s counts half strips if HALF

    // ---- load the block this lane sits on ----
    // Lanes past the matrix' last strip take part in the exchange with a filler block whose start has
    // no excess (a band of ones: entry (i, j) is 1 iff (i + j) mod M < N), so they cost the solver nothing.
    u32x4 raw[M];
    // first byte of the lane's part of row 0 of the block that strip (or half strip) `unit` belongs to
    auto block_base = [&](uint32_t unit) {
        const StripPos pos = strip_pos(md, HALF ? unit >> 1 : unit);
        const size_t col = (size_t)pos.sc * Ge::C + (HALF ? (unit & 1u) * 4u : 0u);
        return (const char *)md.w + ((size_t)pos.br * M * md.ld + col) * Ge::ES;
    };
    auto load_block = [&](bool ok, uint32_t unit) {
#pragma unroll
        for (int i = 0; i < M; i++) {
            uint32_t d[4];
#pragma unroll
            for (int q = 0; q < 4; q++) {
                if constexpr (DT == kF32) {
                    const uint32_t j = gpos * 4u + (uint32_t)q;
                    d[q] = (((uint32_t)i + j) & (M - 1)) < NKEEP ? 0x3F800000u : 0u;
                } else if (HALF && q >= 2) {
                    d[q] = 0u;
                } else {
                    const uint32_t j = gpos * (uint32_t)C + 2u * (uint32_t)q;
                    d[q] = ((((uint32_t)i + j) & (M - 1)) < NKEEP ? 0x3F80u : 0u) |
                           ((((uint32_t)i + j + 1u) & (M - 1)) < NKEEP ? 0x3F800000u : 0u);
                }
            }
            raw[i] = u32x4{d[0], d[1], d[2], d[3]};
        }
        if (ok) {
            const char *base = block_base(unit);
            const size_t row_bytes = (size_t)md.ld * Ge::ES;
#pragma unroll
            for (int i = 0; i < M; i++) {
                if constexpr (PARK) {
                    raw[i] = __builtin_nontemporal_load((const u32x4 *)(base + i * row_bytes));
                } else if constexpr (HALF) {
                    const u32x2 h = *(const u32x2 *)(base + i * row_bytes);
                    raw[i] = u32x4{h.x, h.y, 0u, 0u};
                } else {
                    raw[i] = *(const u32x4 *)(base + i * row_bytes);     // read again below: may stay in the cache
                }
            }
        }
    };
    load_block(valid, s);

    // ---- the solver's start on the block this lane sits on (every lane busy), then a stable counting sort
    //      of the workgroup's blocks by the row excess that start leaves: the number of augmentations to come ----
    uint32_t e = 0;
    {
        uint32_t a[M][C], xcol[C];
        int cost[M][C];
#pragma unroll
        for (int i = 0; i < M; i++) {
            unpack_row<DT, C>(raw[i], a[i]);
            if constexpr (PARK)
                xraw[tid][i] = raw[i];  // parked in LDS for the lane that will run this block's searches
#pragma unroll
            for (int c = 0; c < C; c++)
                asm volatile("" : "+v"(a[i][c]));   // the raw rows end here
        }
        exact_costs<M, C, G>(a, cost);
        e = exact_priced_start<M, C, G, GENERAL>(cost, gpos, xcol, K);
        e = e < (uint32_t)(NBUCKET - 1) ? e : (uint32_t)(NBUCKET - 1);
#pragma unroll
        for (int q = 0; q < XW; q++) {
            uint32_t xp = 0;
#pragma unroll
            for (int c = 0; c < XPW; c++)
                xp |= xcol[q * XPW + c] << (c * M);
            xstart[tid][q] = xp;
        }
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
    ssrc[rank * G + gpos] = (uint16_t)(tid | (e << 8));      // where the block's rows and start are, and its excess
    if (leader)
        sorig[rank] = valid ? s : 0xFFFFFFFFu;
    __syncthreads();

    // ---- this lane continues with the block sorted into its position: rows and start of the lane that loaded it ----
    const uint32_t from = ssrc[tid] & 0xFFu, my_e = ssrc[tid] >> 8;
    const uint32_t my_s = sorig[tid / G];
    const bool my_valid = my_s != 0xFFFFFFFFu;
    if constexpr (PARK) {
#pragma unroll
        for (int i = 0; i < M; i++)
            raw[i] = xraw[from][i];
    } else {
        load_block(my_valid, my_s + gpos);
    }
    uint32_t xpack[XW];
#pragma unroll
    for (int q = 0; q < XW; q++)
        xpack[q] = xstart[from][q];

    // ---- solve ----
    __builtin_amdgcn_sched_barrier(0);
    float acc = 0.f;
    {
        uint32_t a[M][C], xcol[C], bits[M];
#pragma unroll
        for (int i = 0; i < M; i++) {
            unpack_row<DT, C>(raw[i], a[i]);
            // the raw rows end here: the keys must not be re-derived from them later
#pragma unroll
            for (int c = 0; c < C; c++)
                asm volatile("" : "+v"(a[i][c]));
        }
#pragma unroll
        for (int c = 0; c < C; c++)
            xcol[c] = (xpack[c / XPW] >> ((c % XPW) * M)) & ((1u << M) - 1u);
        // most wavefronts hold only blocks whose start is already balanced: nothing to search
        if (__any(my_e != 0u)) {
            int cost[M][C];
            uint32_t cnt[M];
            exact_costs<M, C, G>(a, cost);
            exact_counts<M, C, G>(xcol, cnt);
            (void)exact_phases<M, C, G>(cost, K, gpos, xcol, cnt, M * M);
        }
#pragma unroll
        for (int i = 0; i < M; i++) {
            bits[i] = 0;
#pragma unroll
            for (int c = 0; c < C; c++)
                bits[i] |= (((xcol[c] >> i) & 1u) ^ 1u) << c;
        }
        if (my_valid) {
            const uint32_t unit = my_s + gpos;
            if constexpr (HALF) {
                // four mask entries per row and lane: four bytes, or a nibble that the even lane of a pair completes
                const StripPos pos = strip_pos(md, unit >> 1);
                const size_t col = (size_t)pos.sc * 8u + (unit & 1u) * 4u;
                char *mrow = (char *)md.mask + (size_t)pos.br * M * md.mask_ld;
#pragma unroll
                for (int i = 0; i < M; i++) {
                    if constexpr (FMT == kMaskU8) {
                        stream_store(bits_to_bytes4(bits[i]), (uint32_t *)(mrow + (size_t)i * md.mask_ld + col));
                    } else {
                        const uint32_t other = quad_xor<1>(bits[i]);
                        if ((unit & 1u) == 0)
                            mrow[(size_t)i * md.mask_ld + (col >> 3)] = (char)(bits[i] | (other << 4));
                    }
                }
            } else {
                store_mask<DT, M, FMT>(md, strip_pos(md, unit), bits);
            }
            // the magnitudes are read again (from LDS, or from memory): they need not occupy registers during the solve
            const char *base = block_base(unit);
            const size_t row_bytes = (size_t)md.ld * Ge::ES;
#pragma unroll
            for (int i = 0; i < M; i++) {
                uint32_t ar[C];
                if constexpr (PARK) {
                    unpack_row<DT, C>(xraw[from][i], ar);
                } else if constexpr (HALF) {
                    const u32x2 h = __builtin_nontemporal_load((const u32x2 *)(base + i * row_bytes));
                    unpack_row<DT, C>(u32x4{h.x, h.y, 0u, 0u}, ar);
                } else {
                    unpack_row<DT, C>(__builtin_nontemporal_load((const u32x4 *)(base + i * row_bytes)), ar);
                }
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

// tmask: streaming kernels (approx / exact / score) and the C ABI.  gfx950 only.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <type_traits>
#include <vector>

#include "../../include/tmask.h"
#include "tmask_device.hpp"
#include "tmask_host.hpp"
#include "tmask_solvers.hpp"
#include "tmask_approx4.hpp"
#include "tmask_approx_sel.hpp"
#include "tmask_pack.hpp"
#include "tmask_pack4.hpp"
#include "tmask_pack8.hpp"
#include "tmask_exact_balance.hpp"
#include "tmask_fused4.hpp"

namespace tmask {

// =================================================================================================
// Kernels
// =================================================================================================

enum { kSolveApprox = 0, kSolveExact = 1, kSolveRow1D = 2 };

// One workgroup = 256 consecutive strips of one matrix: load M rows x 16 B per lane, solve the
// block(s) in registers, write the mask, leave one partial objective per workgroup.
template <int SOLVER, int DT, int M, int FMT>
__global__ __launch_bounds__(kThreads) void mask_kernel(const BatchArgs args)
{
    using Ge = Geo<DT, M>;
    __shared__ double red[kThreads / 64];
    const uint32_t tile = blockIdx.x;
    const MatDev md = args.m[find_matrix(args, tile)];
    const uint32_t s = (tile - md.tile0) * kThreads + threadIdx.x;
    const uint32_t gpos = threadIdx.x & (Ge::G - 1);
    float acc = 0.f;
    if (s < md.n_strips) {
        const StripPos pos = strip_pos(md, s);
        uint32_t a[M][Ge::C];
        u32x4 raw[M];
        uint32_t bits[M];
        load_strip<DT, M>(md, pos, a, raw);
        static_assert(SOLVER == kSolveApprox || SOLVER == kSolveRow1D, "the exact solvers have kernels of their own");
        if constexpr (SOLVER == kSolveApprox) {
            approx_keep<DT, M, (M >= 16 && FMT == kMaskBits)>(a, args.K, gpos, bits);
        } else {
            // structured N:M along rows only: an entry is kept iff at least K entries of its group of M
            // precede it in the (magnitude, position) order
            bool done = false;
            if constexpr (DT == kBF16 && M >= 8) {
                if (2u * args.K == (uint32_t)M) {      // N = M/2: thresholds on unique keys instead of pairwise ranks
                    row_half_keep_bf16<M>(raw, gpos, bits);
                    done = true;
                } else if constexpr (M == 8) {         // any N: the sorted row group read at index K
                    row_half_keep_bf16<M, true>(raw, gpos, bits, args.K);
                    done = true;
                }
            }
            if constexpr (DT == kF32 && M == 16) {
                // N = M/2: thresholds on magnitudes (8192^2 8:16: 89 -> 63 us); a wavefront with a cut among equal
                // values falls through to the ranks.  At M = 8 the ranks already run at the speed of the memory.
                if (2u * args.K == (uint32_t)M)
                    done = !__any(row_half_keep_f32<M>(a, gpos, bits));
            }
            if (!done) {
#pragma unroll
                for (int i = 0; i < M; i++)
                    bits[i] = (1u << Ge::C) - 1u;
                row_rank_keep<M, Ge::C, Ge::G, Ge::B, (M >= 16 && FMT == kMaskBits)>(a, args.K, gpos, bits);
            }
        }
        store_mask<DT, M, FMT>(md, pos, bits);
        acc = kept_sum<M, Ge::C>(a, bits);
    }
    if (args.partials) {
        const double t = block_sum_f32(acc, red);
        if (threadIdx.x == 0)
            ((double *)args.partials)[args.partial0 + tile] = t;
    }
}

// tmask_approx for 2:4: same tiling as mask_kernel, decisions taken as lane-mask logic.
template <int DT, int FMT>
__global__ __launch_bounds__(kThreads) void approx24_kernel(const BatchArgs args)
{
    using Ge = Geo<DT, 4>;
    __shared__ double red[kThreads / 64];
    const uint32_t tile = blockIdx.x;
    const MatDev md = args.m[find_matrix(args, tile)];
    const uint32_t s = (tile - md.tile0) * kThreads + threadIdx.x;
    float acc = 0.f;
    if (s < md.n_strips) {
        const StripPos pos = strip_pos(md, s);
        uint32_t a[4][Ge::C];
        u32x4 raw[4];
        load_strip<DT, 4>(md, pos, a, raw);
        acc = approx_2of4_strip<DT, FMT>(md, pos, a);
    }
    if (args.partials) {
        const double t = block_sum_f32(acc, red);
        if (threadIdx.x == 0)
            ((double *)args.partials)[args.partial0 + tile] = t;
    }
}

// tmask_approx for fp32 with N = M/2, M = 8 or 16: thresholds on magnitudes; a wavefront in which some
// line has a tie across its cut redoes its strips with the form that resolves ties by position (uniform branch).
// GENERAL (M = 8): any N, thresholds read from the sorted line; ties send the wavefront to the rank form.
template <int M, int FMT, bool GENERAL = false>
__global__ __launch_bounds__(kThreads, (M == 16 && FMT == kMaskBits) ? 4 : 1) void approx_sel_f32_kernel(const BatchArgs args)
{
    using Ge = Geo<kF32, M>;
    __shared__ double red[kThreads / 64];
    const uint32_t tile = blockIdx.x;
    const MatDev md = args.m[find_matrix(args, tile)];
    const uint32_t s = (tile - md.tile0) * kThreads + threadIdx.x;
    const uint32_t gpos = threadIdx.x & (Ge::G - 1);
    float acc = 0.f;
    if (s < md.n_strips) {
        const StripPos pos = strip_pos(md, s);
        uint32_t a[M][4];
        u32x4 raw[M];
        load_strip<kF32, M>(md, pos, a, raw);
        uint32_t rowbytes[M];
        const bool tie = approx_half_f32<M, GENERAL>(a, gpos, rowbytes, acc, args.K);
        uint32_t bits[M];
        // Some cut among equal values (a matrix full of zeros, say).  M = 8: the form that sorts them out by position
        // (8192^2 with 90 % zeros: 80 -> 60 us).  M = 16: the rank form; the other one takes the kernel from 119 to
        // 154-209 registers whichever way it is attached, which costs the common case more (60 -> 69 us) than it
        // saves here (165 -> 118 us).
        bool stored = false;
        if (__any(tie)) {
            if constexpr (M == 8 && !GENERAL) {
                approx_half_f32_ties<M>(a, gpos, rowbytes, acc);
            } else {
                approx_keep<kF32, M, (M >= 16 && FMT == kMaskBits)>(a, args.K, gpos, bits);
                acc = kept_sum<M, 4>(a, bits);
                if constexpr (FMT == kMaskU8)
                    store_mask<kF32, M, FMT>(md, pos, bits);
                stored = true;
            }
        }
        if constexpr (FMT == kMaskU8) {
            if (!stored) {
                char *mb = (char *)md.mask + (size_t)pos.br * M * md.mask_ld + (size_t)pos.sc * 4;
#pragma unroll
                for (int i = 0; i < M; i++)
                    stream_store(rowbytes[i], (uint32_t *)(mb + (size_t)i * md.mask_ld));
            }
        } else {
            // bit masks leave through one place (the cross-lane assembly of a row's bytes is long code: twice it cost
            // the M = 16 kernel a wavefront of occupancy)
            if (!stored) {
#pragma unroll
                for (int i = 0; i < M; i++)
                    bits[i] = bytes4_to_bits(rowbytes[i]);
            }
            store_mask<kF32, M, kMaskBits>(md, pos, bits);
        }
    }
    if (args.partials) {
        const double t = block_sum_f32(acc, red);
        if (threadIdx.x == 0)
            ((double *)args.partials)[args.partial0 + tile] = t;
    }
}

// tmask_exact at M = 4: every block by enumeration (NK = 2: all 90 patterns; NK = 1, 3: the 24 permutations, kept
// resp. pruned), the kept sum comes with the optimum.
template <int DT, int FMT, int NK = 2>
__global__ __launch_bounds__(kThreads) void exact24_kernel(const BatchArgs args)
{
    using Ge = Geo<DT, 4>;
    __shared__ double red[kThreads / 64];
    const uint32_t tile = blockIdx.x;
    const MatDev md = args.m[find_matrix(args, tile)];
    const uint32_t s = (tile - md.tile0) * kThreads + threadIdx.x;
    float acc = 0.f;
    if (s < md.n_strips) {
        const StripPos pos = strip_pos(md, s);
        uint32_t a[4][Ge::C];
        u32x4 raw[4];
        uint32_t bits[4] = {0u, 0u, 0u, 0u};
        load_strip<DT, 4>(md, pos, a, raw);
        float sum = 0.f;
#pragma unroll
        for (int b = 0; b < Ge::B; b++) {
            float v[4][4];
#pragma unroll
            for (int i = 0; i < 4; i++)
#pragma unroll
                for (int c = 0; c < 4; c++)
                    v[i][c] = __uint_as_float(a[i][b * 4 + c]);
            float best;
            uint32_t m16;
            if constexpr (NK == 2) {
                m16 = exact24_block(v, best);
            } else if constexpr (NK == 1) {
                m16 = best_permutation4<true>(v, best);
            } else {
                m16 = ~best_permutation4<false>(v, best) & 0xFFFFu;
                float all = 0.f;
#pragma unroll
                for (int i = 0; i < 4; i++)
                    all += (v[i][0] + v[i][1]) + (v[i][2] + v[i][3]);
                best = all - best;
            }
            sum += best;
#pragma unroll
            for (int i = 0; i < 4; i++)
                bits[i] |= ((m16 >> (4 * i)) & 0xFu) << (4 * b);
        }
        store_mask<DT, 4, FMT>(md, pos, bits);
        acc = sum;
    }
    if (args.partials) {
        const double t = block_sum_f32(acc, red);
        if (threadIdx.x == 0)
            ((double *)args.partials)[args.partial0 + tile] = t;
    }
}

// tmask_approx for bf16 with N = M/2, M = 8 or 16: thresholds from min/max networks on unique keys.  GENERAL: any N,
// the threshold read from the sorted line at index K = M - N (8192^2 3:8: 40 us; 63 us in the rank form).
template <int M, int FMT, bool GENERAL = false>
__global__ __launch_bounds__(kThreads) void approx_sel_bf16_kernel(const BatchArgs args)
{
    using Ge = Geo<kBF16, M>;
    __shared__ double red[kThreads / 64];
    const uint32_t tile = blockIdx.x;
    const MatDev md = args.m[find_matrix(args, tile)];
    const uint32_t s = (tile - md.tile0) * kThreads + threadIdx.x;
    const uint32_t gpos = threadIdx.x & (Ge::G - 1);
    float acc = 0.f;
    if (s < md.n_strips) {
        const StripPos pos = strip_pos(md, s);
        u32x4 raw[M];
        const char *base = (const char *)md.w + ((size_t)pos.br * M * md.ld + (size_t)pos.sc * 8) * 2;
        const size_t row_bytes = (size_t)md.ld * 2;
#pragma unroll
        for (int i = 0; i < M; i++)
            raw[i] = __builtin_nontemporal_load((const u32x4 *)(base + i * row_bytes));
        if constexpr (FMT == kMaskU8) {
            char *mb = (char *)md.mask + (size_t)pos.br * M * md.mask_ld + (size_t)pos.sc * 8;
            const uint32_t mld = md.mask_ld;
            acc = approx_half_bf16<M, GENERAL>(raw, gpos, [&](int i, uint32_t b0, uint32_t b1) {
                u32x2 v;
                v.x = b0;
                v.y = b1;
                stream_store(v, (u32x2 *)(mb + (size_t)i * mld));
            }, args.K);
        } else {
            uint32_t bits[M];
            acc = approx_half_bf16<M, GENERAL>(raw, gpos, [&](int i, uint32_t b0, uint32_t b1) {
                bits[i] = bytes4_to_bits(b0) | (bytes4_to_bits(b1) << 4);
            }, args.K);
            store_mask<kBF16, M, kMaskBits>(md, pos, bits);
        }
    }
    if (args.partials) {
        const double t = block_sum_f32(acc, red);
        if (threadIdx.x == 0)
            ((double *)args.partials)[args.partial0 + tile] = t;
    }
}

// tmask_approx_dense / tmask_prune_1d_dense: a mask and the masked copy W (.) S in one pass.  Same tiling as the
// kernels above; the keep flags come from the same routines.  MODE: kDenseApprox = Algorithm 1 in the rank form for
// any N, kDenseApproxHalf = Algorithm 1 at N = M/2 (the lane-mask form at M = 4, the threshold networks at M = 8, 16),
// kDenseRow1D = N:M pruning along rows, kDenseRow1DAbsorb = the same with the mean of every row group's pruned
// weights added to its kept ones (Sec. 5; fp32 sums inside the lane in position order, then across the lanes of the
// group pairwise; bf16 results rounded to nearest even).  md.aux = the output matrix, md.pad = its leading dimension
// in elements; the mask is written only if md.mask is not NULL.
// kDenseRow1DHalf / kDenseRow1DHalfAbsorb: the row modes at N = M/2 for bf16 with M = 8, 16, where the row rule is a
// threshold on unique keys (row_half_keep_bf16) and only the raw rows need registers.
enum { kDenseApprox = 0, kDenseApproxHalf = 1, kDenseRow1D = 2, kDenseRow1DAbsorb = 3, kDenseRow1DHalf = 4, kDenseRow1DHalfAbsorb = 5 };

template <int DT, int M, int FMT, int MODE>
__global__ __launch_bounds__(kThreads) void approx_dense_kernel(const BatchArgs args)
{
    constexpr bool HALFN = MODE == kDenseApproxHalf;
    constexpr bool ROWHALF = MODE == kDenseRow1DHalf || MODE == kDenseRow1DHalfAbsorb;
    constexpr bool ABSORB = MODE == kDenseRow1DAbsorb || MODE == kDenseRow1DHalfAbsorb;
    static_assert(!ROWHALF || (DT == kBF16 && M >= 8), "the threshold form of the row rule exists for bf16, M = 8, 16");
    using Ge = Geo<DT, M>;
    constexpr int C = Ge::C, ES = Ge::ES;
    const uint32_t tile = blockIdx.x;
    const MatDev md = args.m[find_matrix(args, tile)];
    const uint32_t s = (tile - md.tile0) * kThreads + threadIdx.x;
    const uint32_t gpos = threadIdx.x & (Ge::G - 1);
    if (s >= md.n_strips)
        return;
    const StripPos pos = strip_pos(md, s);
    uint32_t bits[M];                  // bit c = column c of the lane's strip kept
    u32x4 raw[M];
    constexpr bool GEN8 = MODE == kDenseApprox && DT == kBF16 && M >= 8;   // any N at bf16 M = 8, 16: threshold form too
    if constexpr ((HALFN || ROWHALF || GEN8) && DT == kBF16 && M >= 8) {
        const char *base = (const char *)md.w + ((size_t)pos.br * M * md.ld + (size_t)pos.sc * 8) * 2;
        const size_t row_bytes = (size_t)md.ld * 2;
#pragma unroll
        for (int i = 0; i < M; i++)
            raw[i] = __builtin_nontemporal_load((const u32x4 *)(base + i * row_bytes));
        if constexpr (HALFN || GEN8) {
            (void)approx_half_bf16<M, GEN8>(raw, gpos, [&](int i, uint32_t b0, uint32_t b1) {
                bits[i] = bytes4_to_bits(b0) | (bytes4_to_bits(b1) << 4);
            }, args.K);
        } else {
            row_half_keep_bf16<M>(raw, gpos, bits);
        }
    } else {
        uint32_t a[M][C];
        load_strip<DT, M>(md, pos, a, raw);
        if constexpr (HALFN && M == 4) {
#pragma unroll
            for (int i = 0; i < 4; i++)
                bits[i] = 0;
#pragma unroll
            for (int b = 0; b < C / 4; b++) {
                uint32_t k[4][4], bytes[4];
#pragma unroll
                for (int i = 0; i < 4; i++)
#pragma unroll
                    for (int c = 0; c < 4; c++)
                        k[i][c] = a[i][4 * b + c];
                (void)approx_2of4_block(k, bytes);
#pragma unroll
                for (int i = 0; i < 4; i++)
                    bits[i] |= bytes4_to_bits(bytes[i]) << (4 * b);
            }
        } else if constexpr (HALFN && DT == kF32 && M >= 8) {
            uint32_t rowbytes[M];
            float unused = 0.f;
            const bool tie = approx_half_f32<M>(a, gpos, rowbytes, unused);
            if (__any(tie)) {
                if constexpr (M == 8)
                    approx_half_f32_ties<M>(a, gpos, rowbytes, unused);
                else
                    approx_keep<kF32, M, false>(a, (uint32_t)(M / 2), gpos, bits);
            }
            if (M == 8 || !__any(tie)) {
#pragma unroll
                for (int i = 0; i < M; i++)
                    bits[i] = bytes4_to_bits(rowbytes[i]);
            }
        } else if constexpr (MODE == kDenseRow1D || MODE == kDenseRow1DAbsorb) {
            bool done = false;
            if constexpr (DT == kF32 && M == 16) {
                if (2u * args.K == (uint32_t)M)
                    done = !__any(row_half_keep_f32<M>(a, gpos, bits));
            }
            if (!done) {
#pragma unroll
                for (int i = 0; i < M; i++)
                    bits[i] = (1u << C) - 1u;
                row_rank_keep<M, C, Ge::G, Ge::B, false>(a, args.K, gpos, bits);
            }
        } else {
            approx_keep<DT, M, false>(a, args.K, gpos, bits);
        }
    }
    if (md.mask)
        store_mask<DT, M, FMT>(md, pos, bits);
    char *ob = (char *)md.aux + ((size_t)pos.br * M * md.pad + (size_t)pos.sc * C) * ES;
    const size_t out_row_bytes = (size_t)md.pad * ES;
#pragma unroll
    for (int i = 0; i < M; i++) {
        uint32_t d[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};
        if constexpr (ABSORB) {
            constexpr int S = M < C ? M : C;          // entries of one row group inside the lane
            float v[C];
            if constexpr (DT == kF32) {
#pragma unroll
                for (int c = 0; c < 4; c++)
                    v[c] = __uint_as_float(d[c]);
            } else {
#pragma unroll
                for (int c = 0; c < 4; c++) {
                    v[2 * c] = __uint_as_float(d[c] << 16);
                    v[2 * c + 1] = __uint_as_float(d[c] & 0xFFFF0000u);
                }
            }
#pragma unroll
            for (int g = 0; g < C / S; g++) {
                float ps = 0.f;
                uint32_t pc = 0;
#pragma unroll
                for (int c = g * S; c < (g + 1) * S; c++) {
                    const bool k = (bits[i] >> c) & 1u;
                    ps += k ? 0.f : v[c];
                    pc += k ? 0u : 1u;
                }
                if constexpr (Ge::G >= 2) {
                    ps += __uint_as_float(quad_xor<1>(__float_as_uint(ps)));
                    pc += quad_xor<1>(pc);
                }
                if constexpr (Ge::G == 4) {
                    ps += __uint_as_float(quad_xor<2>(__float_as_uint(ps)));
                    pc += quad_xor<2>(pc);
                }
                const float mean = (pc != 0u && pc != (uint32_t)M) ? ps / (float)pc : 0.f;
#pragma unroll
                for (int c = g * S; c < (g + 1) * S; c++)
                    v[c] = ((bits[i] >> c) & 1u) ? v[c] + mean : 0.f;
            }
            if constexpr (DT == kF32) {
#pragma unroll
                for (int c = 0; c < 4; c++)
                    d[c] = __float_as_uint(v[c]);
            } else {
                typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
                typedef float f32x2 __attribute__((ext_vector_type(2)));
#pragma unroll
                for (int c = 0; c < 4; c++) {
                    union { bf16x2 h; uint32_t w; } cv;
                    cv.h = __builtin_convertvector(f32x2{v[2 * c], v[2 * c + 1]}, bf16x2);   // round to nearest even
                    d[c] = cv.w;
                }
            }
        } else {
#pragma unroll
            for (int q = 0; q < 4; q++) {
                if constexpr (DT == kF32)
                    d[q] &= 0u - ((bits[i] >> q) & 1u);
                else
                    d[q] &= ((0u - ((bits[i] >> (2 * q)) & 1u)) & 0xFFFFu) | ((0u - ((bits[i] >> (2 * q + 1)) & 1u)) << 16);
            }
        }
        stream_store(u32x4{d[0], d[1], d[2], d[3]}, (u32x4 *)(ob + i * out_row_bytes));
    }
}

struct ReduceArgs {
    double *objective[kMaxBatch];
    uint32_t tile0[kMaxBatch + 1];
    uint32_t n_mats;
    uint32_t partial0;
    const double *partials;
};

// Second stage of the objective: workgroup m adds the partials of matrix m in a fixed order.  1024 threads: one
// matrix can have hundreds of thousands of partials, and the loop is a chain of load latencies.
constexpr int kReduceThreads = 1024;
constexpr int kReduceThreadsSmall = 256;    // when no matrix of the launch has more than 512 partial results

template <int THREADS>
__global__ __launch_bounds__(THREADS) void objective_reduce_kernel(const ReduceArgs args)
{
    constexpr int kReduceThreads = THREADS;           // shadows the file-scope constant inside this kernel
    __shared__ double red[kReduceThreads / 64];
    const uint32_t m = blockIdx.x;
    double *dst = args.objective[m];
    if (!dst)
        return;
    // four independent partial sums per thread keep several loads in flight; the order of additions is fixed
    const uint32_t t0 = args.tile0[m], t1 = args.tile0[m + 1];
    const double *src = args.partials + args.partial0;
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    uint32_t t = t0 + threadIdx.x;
    for (; t + 7 * kReduceThreads < t1; t += 8 * kReduceThreads) {
        const double v0 = src[t], v1 = src[t + kReduceThreads], v2 = src[t + 2 * kReduceThreads], v3 = src[t + 3 * kReduceThreads];
        const double v4 = src[t + 4 * kReduceThreads], v5 = src[t + 5 * kReduceThreads], v6 = src[t + 6 * kReduceThreads],
                     v7 = src[t + 7 * kReduceThreads];
        a0 += v0; a1 += v1; a2 += v2; a3 += v3;
        a0 += v4; a1 += v5; a2 += v6; a3 += v7;
    }
    for (; t + 3 * kReduceThreads < t1; t += 4 * kReduceThreads) {
        a0 += src[t];
        a1 += src[t + kReduceThreads];
        a2 += src[t + 2 * kReduceThreads];
        a3 += src[t + 3 * kReduceThreads];
    }
    for (; t < t1; t += kReduceThreads)
        a0 += src[t];
    const double w = wave_sum((a0 + a1) + (a2 + a3));
    if ((threadIdx.x & 63) == 0)
        red[threadIdx.x >> 6] = w;
    __syncthreads();
    if (threadIdx.x == 0) {
        double total = red[0];
#pragma unroll
        for (int k = 1; k < kReduceThreads / 64; k++)
            total += red[k];
        dst[0] = total;
    }
}

// One workgroup per matrix; 256 threads instead of 1024 when every matrix has at most 512 partial results.
static void enqueue_objective_reduce(const ReduceArgs &rargs, int nb, hipStream_t stream)
{
    uint32_t most = 0;
    for (int k = 0; k < nb; k++)
        most = rargs.tile0[k + 1] - rargs.tile0[k] > most ? rargs.tile0[k + 1] - rargs.tile0[k] : most;
    if (most <= 2 * kReduceThreadsSmall)
        hipLaunchKernelGGL(objective_reduce_kernel<kReduceThreadsSmall>, dim3(nb), dim3(kReduceThreadsSmall), 0, stream, rargs);
    else
        hipLaunchKernelGGL(objective_reduce_kernel<kReduceThreads>, dim3(nb), dim3(kReduceThreads), 0, stream, rargs);
}

// Score of a bf16 strip at M = 4 with byte masks (4 rows x 8 columns = two blocks per lane) in packed arithmetic: the
// mask bytes of a row group are normalised to 0x80 / 0x00 once, column counts are byte-wise sums, row counts popcounts
// packed one per byte, "more than N" / "not N" are byte-wise tests followed by a popcount, and the sums run two
// magnitudes at a time through the bf16 dot-product instruction against (1, 1), pruned entries cleared to +0 first
// (a select, so a pruned Inf or NaN does not reach the sum).  About 5 vector instructions per weight instead of 15,
// which matters because bf16 leaves 18 to 24 per weight at HBM speed.
typedef __bf16 score_bf16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float dot2_ones(uint32_t pair, float acc)
{
    union { uint32_t u; score_bf16x2 v; } a, o;
    a.u = pair;
    o.u = 0x3F803F80u;
    return __builtin_amdgcn_fdot2_f32_bf16(a.v, o.v, acc, false);
}

__device__ __forceinline__ uint32_t bytes_nonzero(uint32_t v)      // 0x80 in every byte of v that is not zero
{
    return (((v & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | v) & 0x80808080u;
}

__device__ __forceinline__ void score_strip_bf16_m4(const MatDev &md, StripPos pos, uint32_t N, float &retained, float &total,
                                                    uint32_t &kept, uint32_t &rowv, uint32_t &colv, uint32_t &rowne,
                                                    uint32_t &colne)
{
    const char *base = (const char *)md.w + ((size_t)pos.br * 4 * md.ld + (size_t)pos.sc * 8) * 2;
    const size_t row_bytes = (size_t)md.ld * 2;
    const char *mb = (const char *)md.mask + (size_t)pos.br * 4 * md.mask_ld + (size_t)pos.sc * 8;
    u32x4 raw[4];
    u32x2 mk[4];
#pragma unroll
    for (int i = 0; i < 4; i++) {
        raw[i] = __builtin_nontemporal_load((const u32x4 *)(base + i * row_bytes));
        mk[i] = __builtin_nontemporal_load((const u32x2 *)(mb + (size_t)i * md.mask_ld));
    }
    const uint32_t nrep = N * 0x01010101u;
    float blk[2] = {0.f, 0.f}, tot = 0.f;
    uint32_t colsum[2] = {0u, 0u}, rowpk[2] = {0u, 0u};     // kept per column / per row of a block, one count per byte
#pragma unroll
    for (int i = 0; i < 4; i++) {
#pragma unroll
        for (int b = 0; b < 2; b++) {
            const uint32_t nz = bytes_nonzero(b ? mk[i].y : mk[i].x);
            const uint32_t one = nz >> 7;
            colsum[b] += one;
            rowpk[b] |= (uint32_t)__builtin_popcount(nz) << (8 * i);
            const uint32_t ff = (nz - one) | nz;                                   // 0xFF in every kept byte
            const uint32_t lo = __builtin_amdgcn_perm(ff, ff, 0x01010000u);        // columns 0, 1 as 16-bit masks
            const uint32_t hi = __builtin_amdgcn_perm(ff, ff, 0x03030202u);        // columns 2, 3
            const uint32_t d0 = (b ? raw[i].z : raw[i].x) & 0x7FFF7FFFu;
            const uint32_t d1 = (b ? raw[i].w : raw[i].y) & 0x7FFF7FFFu;
            tot = dot2_ones(d0, tot);
            tot = dot2_ones(d1, tot);
            blk[b] = dot2_ones(d0 & lo, blk[b]);
            blk[b] = dot2_ones(d1 & hi, blk[b]);
        }
    }
    // counts are at most 4 and N at most 3: byte + (0x7F - N) has its top bit set exactly when the count exceeds N
    auto over = [&](uint32_t c) { return (uint32_t)__builtin_popcount((c + (0x7F7F7F7Fu - nrep)) & 0x80808080u); };
    auto differ = [&](uint32_t c) { return (uint32_t)__builtin_popcount(bytes_nonzero(c ^ nrep)); };
#pragma unroll
    for (int b = 0; b < 2; b++) {
        kept += __builtin_amdgcn_sad_u8(colsum[b], 0u, 0u);
        colv += over(colsum[b]);
        colne += differ(colsum[b]);
        rowv += over(rowpk[b]);
        rowne += differ(rowpk[b]);
    }
    if (md.aux) {   // the lane's two per-block sums are neighbours in memory; streamed, not left dirty in the caches
        u32x2 o;
        o.x = __float_as_uint(blk[0]);
        o.y = __float_as_uint(blk[1]);
        float *dst = (float *)md.aux + (size_t)pos.br * (md.spr * 2u) + pos.sc * 2u;
        if (((uintptr_t)dst & 7u) == 0u) {
            stream_store(o, (u32x2 *)dst);
        } else {
            stream_store(o.x, (uint32_t *)dst);
            stream_store(o.y, (uint32_t *)dst + 1);
        }
    }
    retained = blk[0] + blk[1];
    total = tot;
}

template <int DT, int M, int FMT>
__global__ __launch_bounds__(kThreads) void score_kernel(const BatchArgs args)
{
    using Ge = Geo<DT, M>;
    constexpr int C = Ge::C, CL = Ge::CL;
    __shared__ double redd[kThreads / 64][2];
    __shared__ uint32_t redu[kThreads / 64][5];
    const uint32_t tile = blockIdx.x;
    const MatDev md = args.m[find_matrix(args, tile)];
    const uint32_t s = (tile - md.tile0) * kThreads + threadIdx.x;
    const uint32_t gpos = threadIdx.x & (Ge::G - 1);
    const uint32_t N = args.N;
    float retained = 0.f, total = 0.f;
    uint32_t kept = 0, rowv = 0, colv = 0, rowne = 0, colne = 0;
    if constexpr (DT == kBF16 && M == 4 && FMT == kMaskU8) {
        if (s < md.n_strips)
            score_strip_bf16_m4(md, strip_pos(md, s), N, retained, total, kept, rowv, colv, rowne, colne);
    } else if (M >= 16 && s < md.n_strips) {
        // M = 16 (one block per lane group, B = 1): a row at a time, so that only the raw rows and the mask bits stay
        // in registers (with every magnitude unpacked up front the bf16 8:16 kernel held 248 registers: two wavefronts
        // per SIMD; now 94, 8192^2 bf16 8:16: 42 -> 39 us).  Same order of additions as below.  At M = 8 the form below is
        // the faster one (it keeps more loads and additions in flight).
        const StripPos pos = strip_pos(md, s);
        u32x4 raw[M];
        uint32_t bits[M];
        const char *base = (const char *)md.w + ((size_t)pos.br * M * md.ld + (size_t)pos.sc * C) * Ge::ES;
        const size_t row_bytes = (size_t)md.ld * Ge::ES;
#pragma unroll
        for (int i = 0; i < M; i++)
            raw[i] = __builtin_nontemporal_load((const u32x4 *)(base + i * row_bytes));
        load_mask<DT, M, FMT>(md, pos, bits);
        // opaque from here on: otherwise every bit test below is rewritten as a test on the intermediate values of the
        // byte-to-bit conversion, all of which then stay in registers
#pragma unroll
        for (int i = 0; i < M; i++)
            asm volatile("" : "+v"(bits[i]));
        float tot = 0.f, blk = 0.f;
        uint32_t colcnt[C];
#pragma unroll
        for (int c = 0; c < C; c++)
            colcnt[c] = 0;
#pragma unroll
        for (int i = 0; i < M; i++) {
            u32x4 r = raw[i];
            asm volatile("" : "+v"(r.x), "+v"(r.y), "+v"(r.z), "+v"(r.w));    // unpack here, not ahead of the loop
            const uint32_t d[4] = {r.x, r.y, r.z, r.w};
            float m[C];
            if constexpr (DT == kF32) {
#pragma unroll
                for (int c = 0; c < 4; c++)
                    m[c] = __uint_as_float(d[c] & 0x7FFFFFFFu);
            } else {
#pragma unroll
                for (int c = 0; c < 4; c++) {
                    m[2 * c] = __uint_as_float((d[c] << 16) & 0x7FFF0000u);
                    m[2 * c + 1] = __uint_as_float(d[c] & 0x7FFF0000u);
                }
            }
            uint32_t cnt = __builtin_popcount(bits[i] & ((1u << C) - 1u));
            if constexpr (Ge::G >= 2)
                cnt = quad_xor_sum<1>(cnt);
            if constexpr (Ge::G == 4)
                cnt = quad_xor_sum<2>(cnt);
            if (gpos == 0) {
                rowv += cnt > N ? 1u : 0u;
                rowne += cnt != N ? 1u : 0u;
            }
#pragma unroll
            for (int c = 0; c < C; c++) {
                const bool k = (bits[i] >> c) & 1u;
                tot += m[c];
                blk += k ? m[c] : 0.f;
                colcnt[c] += k ? 1u : 0u;
            }
            // the row's contributions are added here and now (left alone, the additions sink to the end of the kernel
            // and every magnitude stays in a register until then)
            asm volatile("" : "+v"(tot), "+v"(blk), "+v"(rowv), "+v"(rowne));
#pragma unroll
            for (int c = 0; c < C; c++)
                asm volatile("" : "+v"(colcnt[c]));
        }
        total = tot;
        retained = blk;
#pragma unroll
        for (int c = 0; c < C; c++) {
            kept += colcnt[c];
            colv += colcnt[c] > N ? 1u : 0u;
            colne += colcnt[c] != N ? 1u : 0u;
        }
        if constexpr (Ge::G >= 2)
            blk += __uint_as_float(quad_xor<1>(__float_as_uint(blk)));
        if constexpr (Ge::G == 4)
            blk += __uint_as_float(quad_xor<2>(__float_as_uint(blk)));
        if (md.aux && gpos == 0) {
            const uint32_t bpr = md.spr / Ge::G;        // blocks per block-row
            stream_store(blk, (float *)md.aux + (size_t)pos.br * bpr + pos.sc / Ge::G);
        }
    } else if (s < md.n_strips) {
        const StripPos pos = strip_pos(md, s);
        uint32_t a[M][C];
        u32x4 raw[M];
        uint32_t bits[M];
        load_strip<DT, M>(md, pos, a, raw);
        load_mask<DT, M, FMT>(md, pos, bits);
        float tot = 0.f;
#pragma unroll
        for (int i = 0; i < M; i++)
#pragma unroll
            for (int c = 0; c < C; c++)
                tot += __uint_as_float(a[i][c]);
        total = tot;
        // columns: lane-local
#pragma unroll
        for (int c = 0; c < C; c++) {
            uint32_t cnt = 0;
#pragma unroll
            for (int i = 0; i < M; i++)
                cnt += (bits[i] >> c) & 1u;
            kept += cnt;
            colv += cnt > N ? 1u : 0u;
            colne += cnt != N ? 1u : 0u;
        }
        // rows: per block inside the lane, summed over the G lanes of the block, counted once
#pragma unroll
        for (int b = 0; b < Ge::B; b++) {
            float blk = 0.f;
#pragma unroll
            for (int i = 0; i < M; i++) {
                uint32_t cnt = __builtin_popcount((bits[i] >> (b * CL)) & ((1u << CL) - 1u));
                if constexpr (Ge::G >= 2)
                    cnt += quad_xor<1>(cnt);
                if constexpr (Ge::G == 4)
                    cnt += quad_xor<2>(cnt);
                if (gpos == 0) {
                    rowv += cnt > N ? 1u : 0u;
                    rowne += cnt != N ? 1u : 0u;
                }
#pragma unroll
                for (int c = 0; c < CL; c++)
                    blk += ((bits[i] >> (b * CL + c)) & 1u) ? __uint_as_float(a[i][b * CL + c]) : 0.f;
            }
            retained += blk;
            if constexpr (Ge::G >= 2)
                blk += __uint_as_float(quad_xor<1>(__float_as_uint(blk)));
            if constexpr (Ge::G == 4)
                blk += __uint_as_float(quad_xor<2>(__float_as_uint(blk)));
            if (md.aux && gpos == 0) {
                // block index inside the matrix: block-row-major
                const uint32_t bpr = md.spr * Ge::B / Ge::G;
                const uint32_t bc = pos.sc * Ge::B / Ge::G + b;
                stream_store(blk, (float *)md.aux + (size_t)pos.br * bpr + bc);
            }
        }
    }
    // One reduction pass: fp32 / packed 32-bit counts inside a wavefront (a lane contributes at most
    // 128 kept, 16 row events and 8 column events, so 16-bit fields cannot overflow over 64 lanes),
    // then the four wavefronts in fp64 / 64-bit through LDS.
    const float w_ret = wave_sum(retained), w_tot = wave_sum(total);
    const uint32_t w_a = wave_sum(kept | (rowv << 16));
    const uint32_t w_b = wave_sum(colv | (colne << 16));
    const uint32_t w_c = wave_sum(rowne);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) {
        redd[wave][0] = (double)w_ret;
        redd[wave][1] = (double)w_tot;
        redu[wave][0] = w_a & 0xFFFFu;
        redu[wave][1] = w_a >> 16;
        redu[wave][2] = w_b & 0xFFFFu;
        redu[wave][3] = w_c;
        redu[wave][4] = w_b >> 16;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        ScorePartial *out = (ScorePartial *)args.partials + args.partial0 + tile;
        double r0 = 0.0, r1 = 0.0;
        unsigned long long u[5] = {0, 0, 0, 0, 0};
#pragma unroll
        for (int k = 0; k < kThreads / 64; k++) {
            r0 += redd[k][0];
            r1 += redd[k][1];
#pragma unroll
            for (int q = 0; q < 5; q++)
                u[q] += redu[k][q];
        }
        out->retained = r0; out->total = r1;
        out->kept = u[0]; out->rowv = u[1]; out->colv = u[2]; out->rowne = u[3]; out->colne = u[4];
    }
}

struct ScoreReduceArgs {
    uint32_t tile0[kMaxBatch + 1];
    uint32_t n_mats;
    uint32_t partial0;
    const ScorePartial *partials;
    tmask_score_out *out;   // entry of the first matrix of this launch
};

// 1024 threads, two records in flight per thread: the loop is a chain of load latencies.  A matrix of 16384 x 16384
// leaves 32768 (bf16) or 65536 (fp32) records, which one workgroup still needs 24 / 41 us for, so large matrices are
// reduced in two launches: STAGE 1, workgroup (m, s) adds slice s of matrix m's records and leaves the sum in the
// slice's first record (only this workgroup reads the slice); STAGE 2, workgroup m adds those first records.
// STAGE 0 is the single launch: workgroup m adds all records of matrix m.
constexpr uint32_t kReduceSlices = 32;
constexpr uint32_t kReduceTwoStageFrom = 8192;    // records of the largest matrix of a launch

// THREADS: 1024, or 256 when no matrix of the launch has more than 512 records (a batch of ordinary layers): four
// wavefronts to start, reduce and add up instead of sixteen.
template <int STAGE, int THREADS = kReduceThreads>
__global__ __launch_bounds__(THREADS) void score_reduce_kernel(const ScoreReduceArgs args)
{
    constexpr uint32_t kReduceThreads = THREADS;      // shadows the file-scope constant inside this kernel
    __shared__ double redd[2][kReduceThreads / 64];
    __shared__ unsigned long long redu[5][kReduceThreads / 64];
    const uint32_t m = blockIdx.x;
    double retained = 0.0, total = 0.0;
    unsigned long long kept = 0, rowv = 0, colv = 0, rowne = 0, colne = 0;
    const uint32_t t0 = args.tile0[m], t1 = args.tile0[m + 1];
    const uint32_t len = (t1 - t0 + kReduceSlices - 1) / kReduceSlices;     // records per slice
    // records base + i * stride, i < count
    uint32_t base = t0, count = t1 - t0, stride = 1;
    if constexpr (STAGE == 1) {
        base = t0 + blockIdx.y * len;
        if (base >= t1)
            return;                                   // the whole workgroup: nothing in this slice
        count = t1 - base < len ? t1 - base : len;
    } else if constexpr (STAGE == 2) {
        stride = len;
        count = len ? (t1 - t0 + len - 1) / len : 0;
    }
    const ScorePartial *src = args.partials + args.partial0 + base;
    uint32_t i = threadIdx.x;
    for (; i + kReduceThreads < count; i += 2 * kReduceThreads) {
        const ScorePartial p = src[(size_t)i * stride];
        const ScorePartial q = src[(size_t)(i + kReduceThreads) * stride];
        retained += p.retained; total += p.total;
        kept += p.kept; rowv += p.rowv; colv += p.colv; rowne += p.rowne; colne += p.colne;
        retained += q.retained; total += q.total;
        kept += q.kept; rowv += q.rowv; colv += q.colv; rowne += q.rowne; colne += q.colne;
    }
    for (; i < count; i += kReduceThreads) {
        const ScorePartial p = src[(size_t)i * stride];
        retained += p.retained; total += p.total;
        kept += p.kept; rowv += p.rowv; colv += p.colv; rowne += p.rowne; colne += p.colne;
    }
    // all seven sums per wavefront first, one barrier, then thread 0 adds the wavefronts in a fixed order
    const double d[2] = {wave_sum(retained), wave_sum(total)};
    const unsigned long long u[5] = {wave_sum(kept), wave_sum(rowv), wave_sum(colv), wave_sum(rowne), wave_sum(colne)};
    if ((threadIdx.x & 63) == 0) {
        const uint32_t w = threadIdx.x >> 6;
#pragma unroll
        for (int k = 0; k < 2; k++)
            redd[k][w] = d[k];
#pragma unroll
        for (int k = 0; k < 5; k++)
            redu[k][w] = u[k];
    }
    __syncthreads();          // every thread's records have arrived by now: STAGE 1 may overwrite the slice's first one
    if (threadIdx.x == 0) {
        double r[2];
        unsigned long long c[5];
#pragma unroll
        for (int k = 0; k < 2; k++) {
            r[k] = redd[k][0];
            for (int w = 1; w < (int)(kReduceThreads / 64); w++)
                r[k] += redd[k][w];
        }
#pragma unroll
        for (int k = 0; k < 5; k++) {
            c[k] = redu[k][0];
            for (int w = 1; w < (int)(kReduceThreads / 64); w++)
                c[k] += redu[k][w];
        }
        if constexpr (STAGE == 1) {
            ScorePartial *o = const_cast<ScorePartial *>(src);
            o->retained = r[0]; o->total = r[1];
            o->kept = c[0]; o->rowv = c[1]; o->colv = c[2]; o->rowne = c[3]; o->colne = c[4];
        } else {
            tmask_score_out *o = args.out + m;
            o->retained_l1 = r[0]; o->total_l1 = r[1];
            o->kept = c[0]; o->row_violations = c[1]; o->col_violations = c[2]; o->row_not_n = c[3]; o->col_not_n = c[4];
        }
    }
}

// =================================================================================================
// Host side
// =================================================================================================

static thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

static bool valid_nm(int N, int M) { return (M == 4 || M == 8 || M == 16 || M == 32) && N > 0 && N < M; }

static size_t elem_size(int dt) { return dt == TMASK_F32 ? 4 : 2; }

// s / d == (uint64(s) * mul) >> shift for every s < 2^31 (d >= 1).
static void magic_div(uint32_t d, uint32_t *mul, uint32_t *shift)
{
    uint32_t l = 0;
    while ((1ull << l) < d)
        l++;
    const uint32_t k = 31 + l;
    *mul = (uint32_t)(((1ull << k) / d) + 1);
    *shift = k;
}

struct HostMat {
    const void *w; int64_t rows, cols, ld;
    void *mask; int64_t mask_ld;
    double *objective;
};

// Validates one matrix for (dt, N, M, mf).  *aligned is cleared (never set) when the matrix misses what the strip
// kernels read and write with -- w 16-byte aligned with ld and cols multiples of 16 bytes, a U8 mask and its pitch
// multiples of the strip width -- in which case the call runs on the column-per-lane kernels instead.
static int check_mat(const HostMat &h, int idx, int dt, int M, int mf, bool need_mask, bool *aligned)
{
    const size_t es = elem_size(dt);
    const int64_t C = 16 / (int64_t)es;
    if (!h.w || (need_mask && !h.mask))
        return fail(TMASK_ERR_NULL, "matrix %d: w or mask is NULL", idx);
    if (h.rows <= 0 || h.cols <= 0 || h.rows % M || h.cols % M || h.ld < h.cols)
        return fail(TMASK_ERR_SHAPE, "matrix %d: rows=%lld cols=%lld ld=%lld must be positive multiples of M=%d with ld >= cols",
                    idx, (long long)h.rows, (long long)h.cols, (long long)h.ld, M);
    if (h.ld > 0x7FFFFFFFll || h.mask_ld > 0x7FFFFFFFll || (h.rows / M) * ((h.cols + 3) / 4) >= 0x7FFFFFFFll)
        return fail(TMASK_ERR_SHAPE, "matrix %d: too large (ld, mask_ld and strip count must stay below 2^31)", idx);
    if ((uintptr_t)h.w % es)
        return fail(TMASK_ERR_ALIGN, "matrix %d: w must be aligned to its element size", idx);
    if (((uintptr_t)h.w & 15) || (h.ld * es) % 16 || (h.cols * es) % 16)
        *aligned = false;
    if (h.mask) {
        if (mf == TMASK_MASK_U8) {
            if (h.mask_ld < h.cols)
                return fail(TMASK_ERR_SHAPE, "matrix %d: mask_ld=%lld < cols", idx, (long long)h.mask_ld);
            if (((uintptr_t)h.mask % C) || (h.mask_ld % C))
                *aligned = false;
        } else {
            if (h.cols % 8)
                return fail(TMASK_ERR_SHAPE, "matrix %d: BITS masks need cols to be a multiple of 8", idx);
            if (h.mask_ld < h.cols / 8)
                return fail(TMASK_ERR_SHAPE, "matrix %d: mask_ld=%lld < cols/8", idx, (long long)h.mask_ld);
        }
    }
    return TMASK_OK;
}

static uint32_t strips_of(const HostMat &h, int dt, int M)
{
    const int64_t C = 16 / (int64_t)elem_size(dt);
    return (uint32_t)((h.rows / M) * (h.cols / C));
}

static uint32_t tiles_of(uint32_t n_strips) { return (n_strips + kThreads - 1) / kThreads; }

static void fill_desc(MatDev &d, const HostMat &h, int dt, int M, uint32_t tile0)
{
    const int64_t C = 16 / (int64_t)elem_size(dt);
    d.w = h.w; d.mask = h.mask; d.aux = nullptr;
    d.ld = (uint32_t)h.ld; d.mask_ld = (uint32_t)h.mask_ld;
    d.spr = (uint32_t)(h.cols / C);
    d.n_strips = strips_of(h, dt, M);
    magic_div(d.spr, &d.div_mul, &d.div_shift);
    d.tile0 = tile0; d.pad = 0;
}

typedef void (*batch_kernel_t)(const BatchArgs);

template <int SOLVER>
static batch_kernel_t pick_mask_kernel(int dt, int M, int mf)
{
#define TMASK_PICK(DT, MM, FM) \
    if (dt == DT && M == MM && mf == FM) return mask_kernel<SOLVER, DT, MM, FM>;
    TMASK_PICK(kF32, 4, kMaskU8) TMASK_PICK(kF32, 8, kMaskU8) TMASK_PICK(kF32, 16, kMaskU8)
    TMASK_PICK(kBF16, 4, kMaskU8) TMASK_PICK(kBF16, 8, kMaskU8) TMASK_PICK(kBF16, 16, kMaskU8)
    TMASK_PICK(kF32, 4, kMaskBits) TMASK_PICK(kF32, 8, kMaskBits) TMASK_PICK(kF32, 16, kMaskBits)
    TMASK_PICK(kBF16, 4, kMaskBits) TMASK_PICK(kBF16, 8, kMaskBits) TMASK_PICK(kBF16, 16, kMaskBits)
#undef TMASK_PICK
    return nullptr;
}

static batch_kernel_t pick_score_kernel(int dt, int M, int mf)
{
#define TMASK_PICK(DT, MM, FM) \
    if (dt == DT && M == MM && mf == FM) return score_kernel<DT, MM, FM>;
    TMASK_PICK(kF32, 4, kMaskU8) TMASK_PICK(kF32, 8, kMaskU8) TMASK_PICK(kF32, 16, kMaskU8)
    TMASK_PICK(kBF16, 4, kMaskU8) TMASK_PICK(kBF16, 8, kMaskU8) TMASK_PICK(kBF16, 16, kMaskU8)
    TMASK_PICK(kF32, 4, kMaskBits) TMASK_PICK(kF32, 8, kMaskBits) TMASK_PICK(kF32, 16, kMaskBits)
    TMASK_PICK(kBF16, 4, kMaskBits) TMASK_PICK(kBF16, 8, kMaskBits) TMASK_PICK(kBF16, 16, kMaskBits)
#undef TMASK_PICK
    return nullptr;
}

static int check_common(const void *mats, int n_mats, int dt, int N, int M, int mf)
{
    if (!mats)
        return fail(TMASK_ERR_NULL, "descriptor array is NULL");
    if (n_mats <= 0)
        return fail(TMASK_ERR_SHAPE, "n_mats=%d must be positive", n_mats);
    if (dt != TMASK_F32 && dt != TMASK_BF16)
        return fail(TMASK_ERR_DTYPE, "unknown dtype %d", dt);
    if (mf != TMASK_MASK_U8 && mf != TMASK_MASK_BITS)
        return fail(TMASK_ERR_DTYPE, "unknown mask format %d", mf);
    if (!valid_nm(N, M))
        return fail(TMASK_ERR_NM, "unsupported N:M = %d:%d (need M in {4,8,16,32}, 0 < N < M)", N, M);
    return TMASK_OK;
}

static size_t workspace_need(const tmask_mat *mats, int n_mats, int M)
{
    // Upper bound over dtypes: fp32 strips (4 columns) are the narrower ones.
    size_t tiles = 0, pack_tiles = 0;
    for (int i = 0; i < n_mats; i++) {
        if (mats[i].rows <= 0 || mats[i].cols <= 0)
            return 0;
        const size_t strips = (size_t)((mats[i].rows + M - 1) / M) * (size_t)((mats[i].cols + 3) / 4);
        // M = 32 runs on the column-per-lane kernels: one partial result per tile of 32 rows x 64 columns
        tiles += M == 32 ? (size_t)((mats[i].rows + 31) / 32) * (size_t)((mats[i].cols + 63) / 64) : (strips + kThreads - 1) / kThreads;
        // tmask_approx_pack keeps one fp64 partial per tile of its one-pass kernels (64 rows x 256 columns at least)
        pack_tiles += (size_t)((mats[i].rows + 63) / 64) * (size_t)((mats[i].cols + 255) / 256);
    }
    const size_t a = tiles * sizeof(ScorePartial), b = pack_tiles * sizeof(double);
    return (a > b ? a : b) + 256;
}

static int check_workspace(const tmask_mat *mats, int n_mats, int M, void *ws, size_t ws_bytes)
{
    if (!ws || ((uintptr_t)ws & 255))
        return fail(TMASK_ERR_WORKSPACE, "workspace is NULL or not 256-byte aligned");
    const size_t need = workspace_need(mats, n_mats, M);
    if (ws_bytes < need)
        return fail(TMASK_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, need);
    return TMASK_OK;
}

int hip_fail(hipError_t e, const char *what)
{
    return fail(TMASK_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

// One-shot profiling events (tmask_profile_next): recorded around the main kernel of the next call.
thread_local hipEvent_t g_prof_start = nullptr, g_prof_stop = nullptr;

// Scratch memory of tmask_approx_noalloc: the per-workgroup partial sums of the objective, which the other entry
// points keep in the caller's workspace.  One copy per GPU, held until the process ends; every call on a GPU shares
// it, so calls that overlap on one GPU race.  Nothing in it has to start at zero: every partial a call reads was
// written by that call.
constexpr size_t kScratchPartials = 65536;      // 512 KiB: one double per workgroup of 256 strips
static __device__ __align__(256) __attribute__((used)) double scratch[kScratchPartials];

constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];        // device address of `scratch` on each GPU (the array's name is only a
static std::mutex g_scratch_lock;               // host-side handle, never a device address)

// Address of the current device's copy of `scratch`, looked up once per device.
static int scratch_of_current_device(void **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices)
        return fail(TMASK_ERR_HIP, "device ordinal %d is outside the %d this library keeps scratch addresses for", dev, kMaxDevices);
    std::lock_guard<std::mutex> guard(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return hip_fail(e, "hipGetSymbolAddress(scratch)");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return TMASK_OK;
}

// own_scratch: the partial sums go to the library's static array instead of a caller workspace (ws, ws_bytes unused).
template <int SOLVER>
static int run_mask(const tmask_mat *mats, int n_mats, int dt, int N, int M, int mf, void *ws, size_t ws_bytes,
                    void *stream_, bool own_scratch = false)
{
    int rc = check_common(mats, n_mats, dt, N, M, mf);
    if (rc)
        return rc;
    bool want_obj = false, aligned = (M != 32);
    for (int i = 0; i < n_mats; i++) {
        const HostMat h{mats[i].w, mats[i].rows, mats[i].cols, mats[i].ld, mats[i].mask, mats[i].mask_ld,
                        mats[i].objective};
        if ((rc = check_mat(h, i, dt, M, mf, true, &aligned)))
            return rc;
        want_obj = want_obj || mats[i].objective;
    }
    if (own_scratch) {
        size_t tiles = 0;
        for (int i = 0; i < n_mats; i++) {
            const HostMat h{mats[i].w, mats[i].rows, mats[i].cols, mats[i].ld, nullptr, 0, nullptr};
            tiles += aligned ? tiles_of(strips_of(h, dt, M)) : cw_workgroups(h.rows, h.cols, M);
        }
        if (want_obj && tiles > kScratchPartials)
            return fail(TMASK_ERR_WORKSPACE,
                        "this call needs %zu partial sums (one per 256 strips of 16 bytes x M rows); the library's own scratch "
                        "array holds %zu: split the batch, or use the entry point that takes a caller workspace",
                        tiles, kScratchPartials);
        if ((rc = scratch_of_current_device(&ws)))
            return rc;
    } else if (want_obj && (rc = check_workspace(mats, n_mats, M, ws, ws_bytes))) {
        return rc;
    }
    // N != M/2 at M = 16, Algorithm 1 and row pruning: the strip kernels have only their rank form there (except
    // Algorithm 1 at bf16, where keys are unique and a row lies in two lanes); the column-per-lane kernels take a
    // threshold from a sorting network
    const bool general_n = 2 * N != M && M == 16 && SOLVER != kSolveExact && !(SOLVER == kSolveApprox && dt == kBF16);
    if (!aligned || general_n)     // also M = 32, or a matrix that the 16-byte strips cannot read
        return cw_run_mask(SOLVER == kSolveApprox ? 0 : SOLVER == kSolveExact ? 1 : 2, mats, n_mats, dt, N, M, mf, ws,
                           (hipStream_t)stream_);
    batch_kernel_t kern = nullptr;
    if constexpr (SOLVER != kSolveExact)      // exact: enumeration at M = 4, the balanced kernel at M = 8, 16 (below)
        kern = pick_mask_kernel<SOLVER>(dt, M, mf);
    if (SOLVER == kSolveApprox && M == 4 && N == 2) {
        if (dt == kF32)
            kern = mf == kMaskU8 ? approx24_kernel<kF32, kMaskU8> : approx24_kernel<kF32, kMaskBits>;
        else
            kern = mf == kMaskU8 ? approx24_kernel<kBF16, kMaskU8> : approx24_kernel<kBF16, kMaskBits>;
    }
    if (SOLVER == kSolveExact && M == 4 && N == 2) {
        if (dt == kF32)
            kern = mf == kMaskU8 ? exact24_kernel<kF32, kMaskU8> : exact24_kernel<kF32, kMaskBits>;
        else
            kern = mf == kMaskU8 ? exact24_kernel<kBF16, kMaskU8> : exact24_kernel<kBF16, kMaskBits>;
    }
    if (SOLVER == kSolveExact && M == 4 && N == 1) {
        if (dt == kF32)
            kern = mf == kMaskU8 ? exact24_kernel<kF32, kMaskU8, 1> : exact24_kernel<kF32, kMaskBits, 1>;
        else
            kern = mf == kMaskU8 ? exact24_kernel<kBF16, kMaskU8, 1> : exact24_kernel<kBF16, kMaskBits, 1>;
    }
    if (SOLVER == kSolveExact && M == 4 && N == 3) {
        if (dt == kF32)
            kern = mf == kMaskU8 ? exact24_kernel<kF32, kMaskU8, 3> : exact24_kernel<kF32, kMaskBits, 3>;
        else
            kern = mf == kMaskU8 ? exact24_kernel<kBF16, kMaskU8, 3> : exact24_kernel<kBF16, kMaskBits, 3>;
    }
    if (SOLVER == kSolveExact && (M == 8 || M == 16)) {
#define TMASK_PICK(DT, MM, FM) \
    if (dt == DT && M == MM && mf == FM) \
        kern = 2 * N == M ? exact_balanced_kernel<DT, MM, FM, false> : exact_balanced_kernel<DT, MM, FM, true>;
        TMASK_PICK(kF32, 8, kMaskU8) TMASK_PICK(kF32, 16, kMaskU8) TMASK_PICK(kBF16, 8, kMaskU8)
        TMASK_PICK(kBF16, 16, kMaskU8) TMASK_PICK(kF32, 8, kMaskBits) TMASK_PICK(kF32, 16, kMaskBits)
        TMASK_PICK(kBF16, 8, kMaskBits) TMASK_PICK(kBF16, 16, kMaskBits)
#undef TMASK_PICK
    }
    if (SOLVER == kSolveApprox && dt == kF32 && M == 8 && N == 4)
        kern = mf == kMaskU8 ? approx_sel_f32_kernel<8, kMaskU8> : approx_sel_f32_kernel<8, kMaskBits>;
    if (SOLVER == kSolveApprox && dt == kF32 && M == 16 && N == 8)
        kern = mf == kMaskU8 ? approx_sel_f32_kernel<16, kMaskU8> : approx_sel_f32_kernel<16, kMaskBits>;
    if (SOLVER == kSolveApprox && dt == kBF16 && M == 16 && N != 8)
        kern = mf == kMaskU8 ? approx_sel_bf16_kernel<16, kMaskU8, true> : approx_sel_bf16_kernel<16, kMaskBits, true>;
    if (SOLVER == kSolveApprox && dt == kF32 && M == 8 && N != 4)
        kern = mf == kMaskU8 ? approx_sel_f32_kernel<8, kMaskU8, true> : approx_sel_f32_kernel<8, kMaskBits, true>;
    if (SOLVER == kSolveApprox && dt == kBF16 && M == 8 && N == 4)
        kern = mf == kMaskU8 ? approx_sel_bf16_kernel<8, kMaskU8> : approx_sel_bf16_kernel<8, kMaskBits>;
    if (SOLVER == kSolveApprox && dt == kBF16 && M == 16 && N == 8)
        kern = mf == kMaskU8 ? approx_sel_bf16_kernel<16, kMaskU8> : approx_sel_bf16_kernel<16, kMaskBits>;
    if (SOLVER == kSolveApprox && dt == kBF16 && M == 8 && N != 4)
        kern = mf == kMaskU8 ? approx_sel_bf16_kernel<8, kMaskU8, true> : approx_sel_bf16_kernel<8, kMaskBits, true>;
    // the exact kernel for bf16 8:16 gives a lane half a strip: twice the workgroups
    const uint32_t unit_split = (SOLVER == kSolveExact && exact_half_strips(dt, M)) ? 2u : 1u;
    hipStream_t stream = (hipStream_t)stream_;
    uint32_t partial0 = 0;
    for (int first = 0; first < n_mats; first += kMaxBatch) {
        const int nb = n_mats - first < kMaxBatch ? n_mats - first : kMaxBatch;
        BatchArgs args;
        ReduceArgs rargs;
        memset(&args, 0, sizeof args);
        memset(&rargs, 0, sizeof rargs);
        uint32_t tiles = 0;
        for (int k = 0; k < nb; k++) {
            const tmask_mat &t = mats[first + k];
            const HostMat h{t.w, t.rows, t.cols, t.ld, t.mask, t.mask_ld, t.objective};
            fill_desc(args.m[k], h, dt, M, tiles);
            rargs.objective[k] = t.objective;
            rargs.tile0[k] = tiles;
            tiles += tiles_of(args.m[k].n_strips * unit_split);
        }
        rargs.tile0[nb] = tiles;
        fill_coarse(args.ci, rargs.tile0, nb, tiles);
        args.n_mats = (uint32_t)nb; args.K = (uint32_t)(M - N); args.N = (uint32_t)N;
        args.partial0 = partial0; args.partials = want_obj ? ws : nullptr;
        {
            ProfileScope prof(stream, first + kMaxBatch >= n_mats);
            hipLaunchKernelGGL(kern, dim3(tiles), dim3(kThreads), 0, stream, args);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return hip_fail(e, "mask kernel launch");
        if (want_obj) {
            rargs.n_mats = (uint32_t)nb; rargs.partial0 = partial0; rargs.partials = (const double *)ws;
            enqueue_objective_reduce(rargs, nb, stream);
            e = hipGetLastError();
            if (e != hipSuccess)
                return hip_fail(e, "objective reduce launch");
        }
        partial0 += tiles;
    }
    return TMASK_OK;
}

// Second-stage reductions for the kernels of other translation units: first0[k] = index (inside this launch) of the
// first partial result of matrix k, first0[nb] = their total number.
int launch_objective_reduce(double *const *objective, const uint32_t *first0, int nb, uint32_t partial0, const void *partials,
                            hipStream_t stream)
{
    ReduceArgs rargs;
    memset(&rargs, 0, sizeof rargs);
    for (int k = 0; k < nb; k++) {
        rargs.objective[k] = objective[k];
        rargs.tile0[k] = first0[k];
    }
    rargs.tile0[nb] = first0[nb];
    rargs.n_mats = (uint32_t)nb; rargs.partial0 = partial0; rargs.partials = (const double *)partials;
    enqueue_objective_reduce(rargs, nb, stream);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? TMASK_OK : hip_fail(e, "objective reduce launch");
}

int launch_score_reduce(const uint32_t *first0, int nb, uint32_t partial0, const void *partials, tmask_score_out *out,
                        hipStream_t stream)
{
    ScoreReduceArgs rargs;
    memset(&rargs, 0, sizeof rargs);
    for (int k = 0; k <= nb; k++)
        rargs.tile0[k] = first0[k];
    rargs.n_mats = (uint32_t)nb; rargs.partial0 = partial0;
    rargs.partials = (const ScorePartial *)partials; rargs.out = out;
    uint32_t most = 0;
    for (int k = 0; k < nb; k++)
        most = first0[k + 1] - first0[k] > most ? first0[k + 1] - first0[k] : most;
    if (most >= kReduceTwoStageFrom) {
        hipLaunchKernelGGL(score_reduce_kernel<1>, dim3(nb, kReduceSlices), dim3(kReduceThreads), 0, stream, rargs);
        hipLaunchKernelGGL(score_reduce_kernel<2>, dim3(nb), dim3(kReduceThreads), 0, stream, rargs);
    } else {
        if (most <= 2 * kReduceThreadsSmall)
            hipLaunchKernelGGL((score_reduce_kernel<0, kReduceThreadsSmall>), dim3(nb), dim3(kReduceThreadsSmall), 0, stream, rargs);
        else
            hipLaunchKernelGGL(score_reduce_kernel<0>, dim3(nb), dim3(kReduceThreads), 0, stream, rargs);
    }
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? TMASK_OK : hip_fail(e, "score reduce launch");
}

}  // namespace tmask

using namespace tmask;

extern "C" {

int tmask_approx(const tmask_mat *mats, int n_mats, tmask_dtype dt, int N, int M, tmask_mask_fmt mf, void *workspace,
                 size_t workspace_bytes, void *hip_stream)
{
    return run_mask<kSolveApprox>(mats, n_mats, (int)dt, N, M, (int)mf, workspace, workspace_bytes, hip_stream);
}

int tmask_approx_noalloc(const tmask_mat *mats, int n_mats, tmask_dtype dt, int N, int M, tmask_mask_fmt mf,
                         void *hip_stream)
{
    return run_mask<kSolveApprox>(mats, n_mats, (int)dt, N, M, (int)mf, nullptr, 0, hip_stream, true);
}

int tmask_prune_1d(const tmask_mat *mats, int n_mats, tmask_dtype dt, int N, int M, tmask_mask_fmt mf, void *workspace,
                   size_t workspace_bytes, void *hip_stream)
{
    return run_mask<kSolveRow1D>(mats, n_mats, (int)dt, N, M, (int)mf, workspace, workspace_bytes, hip_stream);
}

int tmask_exact(const tmask_mat *mats, int n_mats, tmask_dtype dt, int N, int M, tmask_mask_fmt mf, void *workspace,
                size_t workspace_bytes, void *hip_stream)
{
    return run_mask<kSolveExact>(mats, n_mats, (int)dt, N, M, (int)mf, workspace, workspace_bytes, hip_stream);
}

int tmask_score(const tmask_mat *mats, int n_mats, tmask_dtype dt, int N, int M, tmask_mask_fmt mf,
                tmask_score_out *out, float *per_block_obj, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    int rc = check_common(mats, n_mats, (int)dt, N, M, (int)mf);
    if (rc)
        return rc;
    if (!out)
        return fail(TMASK_ERR_NULL, "out is NULL");
    bool aligned = (M != 32);
    for (int i = 0; i < n_mats; i++) {
        const HostMat h{mats[i].w, mats[i].rows, mats[i].cols, mats[i].ld, mats[i].mask, mats[i].mask_ld, nullptr};
        if ((rc = check_mat(h, i, (int)dt, M, (int)mf, true, &aligned)))
            return rc;
    }
    if ((rc = check_workspace(mats, n_mats, M, workspace, workspace_bytes)))
        return rc;
    if (per_block_obj && ((uintptr_t)per_block_obj & 3))
        return fail(TMASK_ERR_ALIGN, "per_block_obj must be 4-byte aligned");
    if (!aligned)
        return cw_run_score(mats, n_mats, (int)dt, N, M, (int)mf, out, per_block_obj, workspace, (hipStream_t)hip_stream);
    const batch_kernel_t kern = pick_score_kernel((int)dt, M, (int)mf);
    hipStream_t stream = (hipStream_t)hip_stream;
    uint32_t partial0 = 0;
    size_t block0 = 0;
    for (int first = 0; first < n_mats; first += kMaxBatch) {
        const int nb = n_mats - first < kMaxBatch ? n_mats - first : kMaxBatch;
        BatchArgs args;
        ScoreReduceArgs rargs;
        memset(&args, 0, sizeof args);
        memset(&rargs, 0, sizeof rargs);
        uint32_t tiles = 0;
        for (int k = 0; k < nb; k++) {
            const tmask_mat &t = mats[first + k];
            const HostMat h{t.w, t.rows, t.cols, t.ld, t.mask, t.mask_ld, nullptr};
            fill_desc(args.m[k], h, (int)dt, M, tiles);
            args.m[k].aux = per_block_obj ? (void *)(per_block_obj + block0) : nullptr;
            block0 += (size_t)(t.rows / M) * (size_t)(t.cols / M);
            rargs.tile0[k] = tiles;
            tiles += tiles_of(args.m[k].n_strips);
        }
        rargs.tile0[nb] = tiles;
        fill_coarse(args.ci, rargs.tile0, nb, tiles);
        args.n_mats = (uint32_t)nb; args.K = (uint32_t)(M - N); args.N = (uint32_t)N;
        args.partial0 = partial0; args.partials = workspace;
        {
            ProfileScope prof(stream, first + kMaxBatch >= n_mats);
            hipLaunchKernelGGL(kern, dim3(tiles), dim3(kThreads), 0, stream, args);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return hip_fail(e, "score kernel launch");
        const int rc = launch_score_reduce(rargs.tile0, nb, partial0, workspace, out + first, stream);
        if (rc)
            return rc;
        partial0 += tiles;
    }
    return TMASK_OK;
}

typedef void (*pack_kernel_t)(const PackArgs);

static pack_kernel_t pick_pack_kernel(int dt, int M, int mf, int N)
{
    if (2 * N == M) {   // N known at compile time
#define TMASK_PICK(DT, MM, FM) \
    if (dt == DT && M == MM && mf == FM) return pack_kernel<DT, MM, FM, MM / 2>;
        TMASK_PICK(kF32, 4, kMaskU8) TMASK_PICK(kF32, 8, kMaskU8) TMASK_PICK(kF32, 16, kMaskU8)
        TMASK_PICK(kBF16, 4, kMaskU8) TMASK_PICK(kBF16, 8, kMaskU8) TMASK_PICK(kBF16, 16, kMaskU8)
        TMASK_PICK(kF32, 4, kMaskBits) TMASK_PICK(kF32, 8, kMaskBits) TMASK_PICK(kF32, 16, kMaskBits)
        TMASK_PICK(kBF16, 4, kMaskBits) TMASK_PICK(kBF16, 8, kMaskBits) TMASK_PICK(kBF16, 16, kMaskBits)
        TMASK_PICK(kF32, 32, kMaskU8) TMASK_PICK(kBF16, 32, kMaskU8) TMASK_PICK(kF32, 32, kMaskBits) TMASK_PICK(kBF16, 32, kMaskBits)
#undef TMASK_PICK
    }
#define TMASK_PICK(DT, MM, FM) \
    if (dt == DT && M == MM && mf == FM) return pack_kernel<DT, MM, FM>;
    TMASK_PICK(kF32, 4, kMaskU8) TMASK_PICK(kF32, 8, kMaskU8) TMASK_PICK(kF32, 16, kMaskU8)
    TMASK_PICK(kBF16, 4, kMaskU8) TMASK_PICK(kBF16, 8, kMaskU8) TMASK_PICK(kBF16, 16, kMaskU8)
    TMASK_PICK(kF32, 4, kMaskBits) TMASK_PICK(kF32, 8, kMaskBits) TMASK_PICK(kF32, 16, kMaskBits)
    TMASK_PICK(kBF16, 4, kMaskBits) TMASK_PICK(kBF16, 8, kMaskBits) TMASK_PICK(kBF16, 16, kMaskBits)
#undef TMASK_PICK
    return nullptr;
}

int tmask_apply_pack(const tmask_pack_desc *descs, int n, tmask_dtype dt, int N, int M, tmask_mask_fmt mf,
                     void *workspace, size_t workspace_bytes, void *hip_stream)
{
    (void)workspace; (void)workspace_bytes;   // this call needs no scratch memory
    int rc = check_common(descs, n, (int)dt, N, M, (int)mf);
    if (rc)
        return rc;
    // M = 32: the tiled kernel at 16:32 (a tile row's position bits are then whole bytes), the column-per-lane one else
    bool aligned = (M != 32) || (N == 16);
    for (int i = 0; i < n; i++) {
        const tmask_pack_desc &p = descs[i];
        const HostMat h{p.w, p.rows, p.cols, p.ld, const_cast<void *>(p.mask), p.mask_ld, nullptr};
        if ((rc = check_mat(h, i, (int)dt, M, (int)mf, true, &aligned)))
            return rc;
        if (!p.vals || !p.idx || !p.valsT || !p.idxT)
            return fail(TMASK_ERR_NULL, "matrix %d: a packed output pointer is NULL", i);
        if (((uintptr_t)p.vals | (uintptr_t)p.valsT) % elem_size((int)dt))
            return fail(TMASK_ERR_ALIGN, "matrix %d: vals and valsT must be aligned to the element size", i);
        if (((uintptr_t)p.vals & 3) || ((uintptr_t)p.valsT & 3))
            aligned = false;
        if (M == 32 && ((uintptr_t)p.vals & 15))     // its row groups leave as 16-byte stores only
            aligned = false;
    }
    if (!aligned)
        return cw_run_pack(descs, n, (int)dt, N, M, (int)mf, (hipStream_t)hip_stream);
    pack_kernel_t kern = pick_pack_kernel((int)dt, M, (int)mf, N);
    uint32_t TC = 256 / (uint32_t)elem_size((int)dt);
    bool fast24 = (M == 4 && N == 2);
    for (int i = 0; i < n && fast24; i++)
        fast24 = (((uintptr_t)descs[i].vals | (uintptr_t)descs[i].valsT) & 7) == 0;
    uint32_t TR = kPackTR, lds_reserve = 0, threads = kThreads;
    if (fast24) {
        // tile widths in strips: measured best per element type (bf16: narrower and taller, so the runs written
        // per column of W^T are 128 bytes long)
        constexpr int SF = 64, SB = 32;
        // four wavefronts working through four block-rows each (eight with two each halves the time a tile stays
        // resident, and measured the same within 1 % at fp32, 8 % slower at bf16)
        constexpr int NW = 4, QN = 4;
        if (dt == TMASK_F32)
            kern = mf == TMASK_MASK_U8 ? pack24_kernel<kF32, kMaskU8, SF, NW, QN> : pack24_kernel<kF32, kMaskBits, SF, NW, QN>;
        else
            kern = mf == TMASK_MASK_U8 ? pack24_kernel<kBF16, kMaskU8, SB, NW, QN> : pack24_kernel<kBF16, kMaskBits, SB, NW, QN>;
        const uint32_t strips = dt == TMASK_F32 ? SF : SB;
        TC = strips * 16 / (uint32_t)elem_size((int)dt);
        TR = 4 * QN * (64 / strips) * NW;
        threads = 64 * NW;
        lds_reserve = dt == TMASK_F32 ? kPack4LdsReservePackF32 : 0;
    }
    bool fast48 = (M == 8 && N == 4 && dt == TMASK_BF16);
    for (int i = 0; i < n && fast48; i++)
        fast48 = (((uintptr_t)descs[i].vals | (uintptr_t)descs[i].valsT) & 7) == 0;
    if (fast48) {
        kern = mf == TMASK_MASK_U8 ? pack48_bf16_kernel<kMaskU8, false, false, PackArgs>
                                   : pack48_bf16_kernel<kMaskBits, false, false, PackArgs>;
        TC = Pack8Geo::TC;
        TR = Pack8Geo::TR;
    }
    bool fast48f = (M == 8 && N == 4 && dt == TMASK_F32);
    for (int i = 0; i < n && fast48f; i++)
        fast48f = (((uintptr_t)descs[i].vals | (uintptr_t)descs[i].valsT) & 7) == 0;
    if (fast48f) {
        kern = mf == TMASK_MASK_U8 ? pack48_f32_kernel<kMaskU8, kPack8F32Strips, false, false, PackArgs>
                                   : pack48_f32_kernel<kMaskBits, kPack8F32Strips, false, false, PackArgs>;
        TC = Pack8F32Geo<kPack8F32Strips>::TC;
        TR = Pack8F32Geo<kPack8F32Strips>::TR;
    }
    hipStream_t stream = (hipStream_t)hip_stream;
    for (int first = 0; first < n; first += kMaxPackBatch) {
        const int nb = n - first < kMaxPackBatch ? n - first : kMaxPackBatch;
        PackArgs args;
        memset(&args, 0, sizeof args);
        uint32_t tiles = 0;
        for (int k = 0; k < nb; k++) {
            const tmask_pack_desc &p = descs[first + k];
            PackDev &d = args.d[k];
            d.w = p.w; d.mask = p.mask; d.vals = p.vals; d.idx = p.idx; d.valsT = p.valsT; d.idxT = p.idxT;
            d.rows = (uint32_t)p.rows; d.cols = (uint32_t)p.cols; d.ld = (uint32_t)p.ld; d.mask_ld = (uint32_t)p.mask_ld;
            d.tiles_x = (d.cols + TC - 1) / TC;
            d.tile0 = tiles;
            tiles += d.tiles_x * ((d.rows + TR - 1) / TR);
        }
        {
            uint32_t first0[kMaxPackBatch + 1];
            for (int k = 0; k < nb; k++)
                first0[k] = args.d[k].tile0;
            first0[nb] = tiles;
            fill_coarse(args.ci, first0, nb, tiles);
        }
        args.n = (uint32_t)nb; args.N = (uint32_t)N;
        {
            ProfileScope prof(stream, first + kMaxPackBatch >= n);
            hipLaunchKernelGGL(kern, dim3(tiles), dim3(threads), lds_reserve, stream, args);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return hip_fail(e, "pack kernel launch");
    }
    return TMASK_OK;
}

int tmask_approx_pack(const tmask_fused_desc *descs, int n, tmask_dtype dt, int N, int M, tmask_mask_fmt mf,
                      void *workspace, size_t workspace_bytes, void *hip_stream)
{
    int rc = check_common(descs, n, (int)dt, N, M, (int)mf);
    if (rc)
        return rc;
    bool fused24 = (M == 4 && N == 2);                         // both need aligned inputs and 8-byte aligned outputs,
    bool fused48 = (M == 8 && N == 4);                         // else the call runs as two steps
    int with_mask = 0;
    bool want_obj = false, aligned = (M != 32);
    for (int i = 0; i < n; i++) {
        const tmask_fused_desc &p = descs[i];
        with_mask += p.mask ? 1 : 0;
        want_obj = want_obj || p.objective;
        const HostMat h{p.w, p.rows, p.cols, p.ld, p.mask, p.mask_ld, p.objective};
        if ((rc = check_mat(h, i, (int)dt, M, (int)mf, p.mask != nullptr, &aligned)))
            return rc;
        if (!p.vals || !p.idx || !p.valsT || !p.idxT)
            return fail(TMASK_ERR_NULL, "matrix %d: a packed output pointer is NULL", i);
        if (((uintptr_t)p.vals | (uintptr_t)p.valsT) % elem_size((int)dt))
            return fail(TMASK_ERR_ALIGN, "matrix %d: vals and valsT must be aligned to the element size", i);
        const bool out8 = ((((uintptr_t)p.vals | (uintptr_t)p.valsT) & 7) == 0);
        fused24 = fused24 && out8;
        fused48 = fused48 && out8;
    }
    const bool fused = aligned && (fused24 || fused48);
    if (with_mask != 0 && with_mask != n)
        return fail(TMASK_ERR_NULL, "mask must be given for all matrices or for none (%d of %d have one)", with_mask, n);
    if (!fused && with_mask == 0)
        return fail(TMASK_ERR_NULL, "this call (N:M = %d:%d, or matrices / outputs that miss the alignment of the one-pass "
                                    "kernels) runs as two steps and needs the mask buffers", N, M);

    if (!fused) {
        std::vector<tmask_mat> mats((size_t)n);
        std::vector<tmask_pack_desc> pds((size_t)n);
        for (int i = 0; i < n; i++) {
            const tmask_fused_desc &p = descs[i];
            mats[i] = tmask_mat{p.w, p.rows, p.cols, p.ld, p.mask, p.mask_ld, p.objective};
            pds[i] = tmask_pack_desc{p.w, p.rows, p.cols, p.ld, p.mask, p.mask_ld, p.vals, p.idx, p.valsT, p.idxT};
        }
        if ((rc = run_mask<kSolveApprox>(mats.data(), n, (int)dt, N, M, (int)mf, workspace, workspace_bytes, hip_stream)))
            return rc;
        return tmask_apply_pack(pds.data(), n, dt, N, M, mf, workspace, workspace_bytes, hip_stream);
    }

    // tile shapes as in tmask_apply_pack
    constexpr int SF = 64, SB = 32;
    const uint32_t strips = dt == TMASK_F32 ? SF : SB;
    using G8F = Pack8F32Geo<kPack8F32Strips>;
    const uint32_t TC = fused48 ? (dt == TMASK_F32 ? (uint32_t)G8F::TC : (uint32_t)Pack8Geo::TC)
                                : strips * 16 / (uint32_t)elem_size((int)dt);
    const uint32_t kPack4Rows = fused48 ? (dt == TMASK_F32 ? (uint32_t)G8F::TR : (uint32_t)Pack8Geo::TR) : 4096 / strips;
    if (want_obj) {
        size_t tiles = 0;
        for (int i = 0; i < n; i++)
            tiles += (size_t)((descs[i].cols + TC - 1) / TC) * (size_t)((descs[i].rows + kPack4Rows - 1) / kPack4Rows);
        if (!workspace || ((uintptr_t)workspace & 255))
            return fail(TMASK_ERR_WORKSPACE, "workspace is NULL or not 256-byte aligned");
        if (workspace_bytes < tiles * sizeof(double))
            return fail(TMASK_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, tiles * sizeof(double));
    }
    typedef void (*fused_kernel_t)(const FusedArgs);
    fused_kernel_t kern = nullptr;
#define TMASK_PICK(DT, FM, SS) \
    if ((int)dt == DT && (int)mf == FM) \
        kern = with_mask ? approx_pack24_kernel<DT, FM, true, SS> : approx_pack24_kernel<DT, FM, false, SS>;
    TMASK_PICK(kF32, kMaskU8, SF) TMASK_PICK(kF32, kMaskBits, SF) TMASK_PICK(kBF16, kMaskU8, SB) TMASK_PICK(kBF16, kMaskBits, SB)
#undef TMASK_PICK
    if (fused48 && dt == TMASK_F32) {
        constexpr int S8 = kPack8F32Strips;
        if (mf == TMASK_MASK_U8)
            kern = with_mask ? pack48_f32_kernel<kMaskU8, S8, true, true, FusedArgs> : pack48_f32_kernel<kMaskU8, S8, true, false, FusedArgs>;
        else
            kern = with_mask ? pack48_f32_kernel<kMaskBits, S8, true, true, FusedArgs>
                             : pack48_f32_kernel<kMaskBits, S8, true, false, FusedArgs>;
    } else if (fused48) {
        if (mf == TMASK_MASK_U8)
            kern = with_mask ? pack48_bf16_kernel<kMaskU8, true, true, FusedArgs> : pack48_bf16_kernel<kMaskU8, true, false, FusedArgs>;
        else
            kern = with_mask ? pack48_bf16_kernel<kMaskBits, true, true, FusedArgs>
                             : pack48_bf16_kernel<kMaskBits, true, false, FusedArgs>;
    }
    hipStream_t stream = (hipStream_t)hip_stream;
    uint32_t partial0 = 0;
    for (int first = 0; first < n; first += kMaxPackBatch) {
        const int nb = n - first < kMaxPackBatch ? n - first : kMaxPackBatch;
        FusedArgs args;
        ReduceArgs rargs;
        memset(&args, 0, sizeof args);
        memset(&rargs, 0, sizeof rargs);
        uint32_t tiles = 0;
        for (int k = 0; k < nb; k++) {
            const tmask_fused_desc &p = descs[first + k];
            PackDev &d = args.d[k];
            d.w = p.w; d.mask = p.mask; d.vals = p.vals; d.idx = p.idx; d.valsT = p.valsT; d.idxT = p.idxT;
            d.rows = (uint32_t)p.rows; d.cols = (uint32_t)p.cols; d.ld = (uint32_t)p.ld; d.mask_ld = (uint32_t)p.mask_ld;
            d.tiles_x = (d.cols + TC - 1) / TC;
            d.tile0 = tiles;
            rargs.objective[k] = p.objective;
            rargs.tile0[k] = tiles;
            tiles += d.tiles_x * ((d.rows + kPack4Rows - 1) / kPack4Rows);
        }
        rargs.tile0[nb] = tiles;
        fill_coarse(args.ci, rargs.tile0, nb, tiles);
        args.n = (uint32_t)nb; args.partial0 = partial0; args.partials = want_obj ? workspace : nullptr;
        {
            ProfileScope prof(stream, first + kMaxPackBatch >= n);
            hipLaunchKernelGGL(kern, dim3(tiles), dim3(kThreads), (fused24 && dt == TMASK_F32) ? kPack4LdsReserveFusedF32 : 0, stream,
                               args);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return hip_fail(e, "fused approx+pack kernel launch");
        if (want_obj) {
            rargs.n_mats = (uint32_t)nb; rargs.partial0 = partial0; rargs.partials = (const double *)workspace;
            enqueue_objective_reduce(rargs, nb, stream);
            e = hipGetLastError();
            if (e != hipSuccess)
                return hip_fail(e, "objective reduce launch");
        }
        partial0 += tiles;
    }
    return TMASK_OK;
}

static int run_mask_dense(const tmask_mask_dense_desc *descs, int n, tmask_dtype dt, int N, int M, tmask_mask_fmt mf,
                          int mode, void *hip_stream)
{
    int rc = check_common(descs, n, (int)dt, N, M, (int)mf);
    if (rc)
        return rc;
    const int64_t es = elem_size((int)dt);
    int with_mask = 0;
    bool aligned = (M != 32);
    for (int i = 0; i < n; i++) {
        const tmask_mask_dense_desc &p = descs[i];
        with_mask += p.mask ? 1 : 0;
        const HostMat h{p.w, p.rows, p.cols, p.ld, p.mask, p.mask_ld, nullptr};
        if ((rc = check_mat(h, i, (int)dt, M, (int)mf, p.mask != nullptr, &aligned)))
            return rc;
        if (!p.out)
            return fail(TMASK_ERR_NULL, "matrix %d: out is NULL", i);
        if (p.ld_out < p.cols || p.ld_out * es > 0x7FFFFFFFll)
            return fail(TMASK_ERR_SHAPE, "matrix %d: ld_out=%lld must cover a row of %lld columns", i, (long long)p.ld_out,
                        (long long)p.cols);
        if ((uintptr_t)p.out % (uintptr_t)es)
            return fail(TMASK_ERR_ALIGN, "matrix %d: out must be aligned to its element size", i);
        if (((uintptr_t)p.out | (uint64_t)(p.ld_out * es)) & 15)
            aligned = false;
    }
    if (with_mask != 0 && with_mask != n)
        return fail(TMASK_ERR_NULL, "mask must be given for all matrices or for none (%d of %d have one)", with_mask, n);
    // Algorithm 1 with N != M/2 at M = 16: the strip kernels have only their rank form there (see run_mask); the
    // row modes are faster on the strips (8192^2 fp32 5:16 with absorption: 101 against 121 us)
    if (!aligned || (2 * N != M && M == 16 && mode == kDenseApprox && dt != kBF16)) {
        const bool absorb = mode == kDenseRow1DAbsorb || mode == kDenseRow1DHalfAbsorb;
        const bool rows_only = absorb || mode == kDenseRow1D || mode == kDenseRow1DHalf;
        return cw_run_dense(descs, n, (int)dt, N, M, (int)mf, absorb ? 2 : rows_only ? 1 : 0, (hipStream_t)hip_stream);
    }
    batch_kernel_t kern = nullptr;
#define TMASK_PICK(DT, MM, FM) \
    if ((int)dt == DT && M == MM && (int)mf == FM) \
        kern = mode == kDenseApprox ? approx_dense_kernel<DT, MM, FM, kDenseApprox> \
             : mode == kDenseApproxHalf ? approx_dense_kernel<DT, MM, FM, kDenseApproxHalf> \
             : mode == kDenseRow1D ? approx_dense_kernel<DT, MM, FM, kDenseRow1D> \
             : mode == kDenseRow1DAbsorb ? approx_dense_kernel<DT, MM, FM, kDenseRow1DAbsorb> : kern;
    TMASK_PICK(kF32, 4, kMaskU8) TMASK_PICK(kF32, 8, kMaskU8) TMASK_PICK(kF32, 16, kMaskU8)
    TMASK_PICK(kBF16, 4, kMaskU8) TMASK_PICK(kBF16, 8, kMaskU8) TMASK_PICK(kBF16, 16, kMaskU8)
    TMASK_PICK(kF32, 4, kMaskBits) TMASK_PICK(kF32, 8, kMaskBits) TMASK_PICK(kF32, 16, kMaskBits)
    TMASK_PICK(kBF16, 4, kMaskBits) TMASK_PICK(kBF16, 8, kMaskBits) TMASK_PICK(kBF16, 16, kMaskBits)
#undef TMASK_PICK
#define TMASK_PICK(MM, FM) \
    if ((int)dt == kBF16 && M == MM && (int)mf == FM && mode >= kDenseRow1DHalf) \
        kern = mode == kDenseRow1DHalf ? approx_dense_kernel<kBF16, MM, FM, kDenseRow1DHalf> \
                                       : approx_dense_kernel<kBF16, MM, FM, kDenseRow1DHalfAbsorb>;
    TMASK_PICK(8, kMaskU8) TMASK_PICK(16, kMaskU8) TMASK_PICK(8, kMaskBits) TMASK_PICK(16, kMaskBits)
#undef TMASK_PICK
    hipStream_t stream = (hipStream_t)hip_stream;
    for (int first = 0; first < n; first += kMaxBatch) {
        const int nb = n - first < kMaxBatch ? n - first : kMaxBatch;
        BatchArgs args;
        memset(&args, 0, sizeof args);
        uint32_t tiles = 0;
        for (int k = 0; k < nb; k++) {
            const tmask_mask_dense_desc &p = descs[first + k];
            const HostMat h{p.w, p.rows, p.cols, p.ld, p.mask, p.mask_ld, nullptr};
            fill_desc(args.m[k], h, (int)dt, M, tiles);
            args.m[k].aux = p.out;
            args.m[k].pad = (uint32_t)p.ld_out;
            tiles += tiles_of(args.m[k].n_strips);
        }
        {
            uint32_t first0[kMaxBatch + 1];
            for (int k = 0; k < nb; k++)
                first0[k] = args.m[k].tile0;
            first0[nb] = tiles;
            fill_coarse(args.ci, first0, nb, tiles);
        }
        args.n_mats = (uint32_t)nb; args.K = (uint32_t)(M - N); args.N = (uint32_t)N;
        {
            ProfileScope prof(stream, first + kMaxBatch >= n);
            hipLaunchKernelGGL(kern, dim3(tiles), dim3(kThreads), 0, stream, args);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return hip_fail(e, "mask + dense copy kernel launch");
    }
    return TMASK_OK;
}

int tmask_approx_dense(const tmask_mask_dense_desc *descs, int n, tmask_dtype dt, int N, int M, tmask_mask_fmt mf,
                       void *hip_stream)
{
    return run_mask_dense(descs, n, dt, N, M, mf, 2 * N == M ? kDenseApproxHalf : kDenseApprox, hip_stream);
}

int tmask_prune_1d_dense(const tmask_mask_dense_desc *descs, int n, tmask_dtype dt, int N, int M, int absorb_mean,
                         tmask_mask_fmt mf, void *hip_stream)
{
    const bool half = dt == TMASK_BF16 && M >= 8 && 2 * N == M;
    const int mode = half ? (absorb_mean ? kDenseRow1DHalfAbsorb : kDenseRow1DHalf)
                          : (absorb_mean ? kDenseRow1DAbsorb : kDenseRow1D);
    return run_mask_dense(descs, n, dt, N, M, mf, mode, hip_stream);
}

size_t tmask_workspace_bytes(const tmask_mat *mats, int n_mats, int N, int M)
{
    if (!mats || n_mats <= 0 || !valid_nm(N, M))
        return 0;
    return workspace_need(mats, n_mats, M);
}

int tmask_profile_next(void *start_event, void *stop_event)
{
    g_prof_start = (hipEvent_t)start_event;
    g_prof_stop = (hipEvent_t)stop_event;
    return TMASK_OK;
}

const char *tmask_last_error(void) { return g_err; }

int tmask_version(void) { return 100; }

}  // extern "C"

// Small companions of the mask kernels: the mask-flip counter of a dynamic-mask training loop, the dense masked
// copy with mean absorption, the pattern-violation counter of Sec. 5, and the mask-diversity formulas (arXiv 2102.08124, Sec. 3, Eq. 2) with the N:M probability of Sec. 5, Eq. 4.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstring>

#include "../../include/tmask.h"
#include "tmask_device.hpp"
#include "tmask_host.hpp"

namespace tmask {

constexpr int kMaxFlipBatch = 256;

struct FlipDev {
    const unsigned char *a, *b;
    unsigned long long *flips;
    uint32_t rows, row_bytes, ld_a, ld_b;   // row_bytes = bytes of a row that carry mask entries
    uint32_t chunks_per_row, wg0;           // chunk = VEC bytes; wg0 = first workgroup of this matrix
    uint32_t n_wg, pad;
};

struct FlipArgs {
    FlipDev d[kMaxFlipBatch];
    uint32_t n;
};
static_assert(sizeof(FlipArgs) <= 16384, "descriptor table is sized to stay a small kernel argument");

__global__ void flip_zero_kernel(const FlipArgs args)
{
    if (threadIdx.x < args.n)
        *args.d[threadIdx.x].flips = 0ull;
}

// differing entries between two runs of VEC mask bytes.  U8: an entry is kept iff its byte is non-zero.
template <int FMT>
__device__ __forceinline__ uint32_t differing(uint32_t x, uint32_t y)
{
    if constexpr (FMT == kMaskBits)
        return (uint32_t)__builtin_popcount(x ^ y);
    else
        return (uint32_t)__builtin_popcount(bytes4_to_bits(x) ^ bytes4_to_bits(y));
}

template <int FMT, int VEC>
__global__ __launch_bounds__(kThreads) void flip_count_kernel(const FlipArgs args)
{
    __shared__ uint32_t red[kThreads / 64];
    int lo = 0, hi = (int)args.n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (args.d[mid].wg0 <= blockIdx.x)
            lo = mid;
        else
            hi = mid - 1;
    }
    const FlipDev d = args.d[lo];
    const uint32_t total = d.rows * d.chunks_per_row;
    uint32_t cnt = 0;
    const uint32_t stride = d.n_wg * kThreads;
    if constexpr (VEC == 16) {
        // a workgroup takes four consecutive runs of 256 chunks per trip (16 KiB of each mask); the four
        // chunk pairs of a lane are independent, so eight 16-byte loads are in flight per lane
        for (uint32_t base = (blockIdx.x - d.wg0) * 4u * kThreads; base < total; base += 4u * stride) {
            u32x4 x[4], y[4];
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const uint32_t c = base + (uint32_t)u * kThreads + threadIdx.x;
                x[u] = y[u] = u32x4{0u, 0u, 0u, 0u};
                if (c < total) {
                    const uint32_t r = c / d.chunks_per_row, j = c - r * d.chunks_per_row;
                    x[u] = __builtin_nontemporal_load((const u32x4 *)(d.a + (size_t)r * d.ld_a + (size_t)j * 16u));
                    y[u] = __builtin_nontemporal_load((const u32x4 *)(d.b + (size_t)r * d.ld_b + (size_t)j * 16u));
                }
            }
#pragma unroll
            for (int u = 0; u < 4; u++)
                cnt += differing<FMT>(x[u].x, y[u].x) + differing<FMT>(x[u].y, y[u].y) + differing<FMT>(x[u].z, y[u].z) +
                       differing<FMT>(x[u].w, y[u].w);
        }
    } else {
        for (uint32_t c = (blockIdx.x - d.wg0) * kThreads + threadIdx.x; c < total; c += stride) {
            const uint32_t r = c / d.chunks_per_row, j = c - r * d.chunks_per_row;
            const unsigned char *pa = d.a + (size_t)r * d.ld_a + (size_t)j * VEC;
            const unsigned char *pb = d.b + (size_t)r * d.ld_b + (size_t)j * VEC;
            if constexpr (VEC == 4)
                cnt += differing<FMT>(*(const uint32_t *)pa, *(const uint32_t *)pb);
            else
                cnt += differing<FMT>((uint32_t)*pa, (uint32_t)*pb);
        }
    }
    const uint32_t t = block_sum(cnt, red);
    if (threadIdx.x == 0 && t)
        atomicAdd(d.flips, (unsigned long long)t);     // integer sum: order does not matter
}

typedef void (*flip_kernel_t)(const FlipArgs);

}  // namespace tmask

using namespace tmask;

extern "C" int tmask_flip_count(const tmask_flip_desc *descs, int n, tmask_mask_fmt mf, void *hip_stream)
{
    if (!descs)
        return fail(TMASK_ERR_NULL, "descriptor array is NULL");
    if (n <= 0)
        return fail(TMASK_ERR_SHAPE, "n=%d must be positive", n);
    if (mf != TMASK_MASK_U8 && mf != TMASK_MASK_BITS)
        return fail(TMASK_ERR_DTYPE, "unknown mask format %d", (int)mf);
    int vec = 16;
    for (int i = 0; i < n; i++) {
        const tmask_flip_desc &f = descs[i];
        if (!f.mask_a || !f.mask_b || !f.flips)
            return fail(TMASK_ERR_NULL, "matrix %d: mask_a, mask_b or flips is NULL", i);
        if (f.rows <= 0 || f.cols <= 0 || (mf == TMASK_MASK_BITS && f.cols % 8))
            return fail(TMASK_ERR_SHAPE, "matrix %d: rows=%lld cols=%lld (BITS masks need cols to be a multiple of 8)", i,
                        (long long)f.rows, (long long)f.cols);
        const int64_t row_bytes = mf == TMASK_MASK_U8 ? f.cols : f.cols / 8;
        if (f.ld_a < row_bytes || f.ld_b < row_bytes || f.ld_a > 0x7FFFFFFFll || f.ld_b > 0x7FFFFFFFll ||
            f.rows * row_bytes >= 0xFFFFFFFFll)
            return fail(TMASK_ERR_SHAPE, "matrix %d: leading dimensions must cover a row; sizes must stay below 2^32 bytes", i);
        if ((uintptr_t)f.flips & 7)
            return fail(TMASK_ERR_ALIGN, "matrix %d: flips must be 8-byte aligned", i);
        // widest load all matrices allow
        const uint64_t bits = (uint64_t)(uintptr_t)f.mask_a | (uint64_t)(uintptr_t)f.mask_b | (uint64_t)f.ld_a |
                              (uint64_t)f.ld_b | (uint64_t)row_bytes;
        while (vec > 1 && (bits & (uint64_t)(vec - 1)))
            vec = vec == 16 ? 4 : 1;
    }
    flip_kernel_t kern;
    if (mf == TMASK_MASK_U8)
        kern = vec == 16 ? flip_count_kernel<kMaskU8, 16> : vec == 4 ? flip_count_kernel<kMaskU8, 4> : flip_count_kernel<kMaskU8, 1>;
    else
        kern = vec == 16 ? flip_count_kernel<kMaskBits, 16> : vec == 4 ? flip_count_kernel<kMaskBits, 4> : flip_count_kernel<kMaskBits, 1>;
    hipStream_t stream = (hipStream_t)hip_stream;
    for (int first = 0; first < n; first += kMaxFlipBatch) {
        const int nb = n - first < kMaxFlipBatch ? n - first : kMaxFlipBatch;
        FlipArgs args;
        memset(&args, 0, sizeof args);
        uint32_t wgs = 0;
        for (int k = 0; k < nb; k++) {
            const tmask_flip_desc &f = descs[first + k];
            FlipDev &d = args.d[k];
            const int64_t row_bytes = mf == TMASK_MASK_U8 ? f.cols : f.cols / 8;
            d.a = (const unsigned char *)f.mask_a; d.b = (const unsigned char *)f.mask_b;
            d.flips = (unsigned long long *)f.flips;
            d.rows = (uint32_t)f.rows; d.row_bytes = (uint32_t)row_bytes;
            d.ld_a = (uint32_t)f.ld_a; d.ld_b = (uint32_t)f.ld_b;
            d.chunks_per_row = (uint32_t)(row_bytes / vec);
            const uint64_t chunks = (uint64_t)d.rows * d.chunks_per_row;
            // 4 chunks per thread and trip, at least one workgroup, at most 1024 per matrix: every workgroup
            // ends with one atomic add on the matrix' counter, and thousands of those on one address cost
            // more than the streaming itself
            uint64_t nw = (chunks + 4ull * kThreads - 1) / (4ull * kThreads);
            nw = nw < 1 ? 1 : nw > 1024 ? 1024 : nw;
            d.n_wg = (uint32_t)nw; d.wg0 = wgs;
            wgs += d.n_wg;
        }
        args.n = (uint32_t)nb;
        hipLaunchKernelGGL(flip_zero_kernel, dim3(1), dim3(kMaxFlipBatch), 0, stream, args);
        {
            ProfileScope prof(stream, first + kMaxFlipBatch >= n);
            hipLaunchKernelGGL(kern, dim3(wgs), dim3(kThreads), 0, stream, args);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return hip_fail(e, "flip count launch");
    }
    return TMASK_OK;
}

// ---------------------------------------------------------------------------------------------------------
// Dense masked copy (Sec. 4) with the optional mean absorption of Sec. 5.
// ---------------------------------------------------------------------------------------------------------
namespace tmask {

constexpr int kMaxDenseBatch = 256;

struct DenseDev {
    const char *w;
    const unsigned char *mask;
    char *out;
    uint32_t rows, chunks_per_row;          // chunk = 16 bytes of a row of W
    uint32_t ld_b, ld_out_b, mask_ld;       // leading dimensions in bytes
    uint32_t wg0, n_wg, pad;
};

struct DenseArgs {
    DenseDev d[kMaxDenseBatch];
    uint32_t n;
};
static_assert(sizeof(DenseArgs) <= 16384, "descriptor table is sized to stay a small kernel argument");

// A lane owns 16 bytes of a row: C = 4 (fp32) or 8 (bf16) entries.  A group of M entries is either a part of
// the lane's chunk (M <= C) or spans G = M / C neighbouring lanes, whose partial sums meet in a butterfly.
template <int DT, int FMT, int M, bool ABSORB>
__global__ __launch_bounds__(kThreads) void apply_dense_kernel(const DenseArgs args)
{
    constexpr int C = DT == kF32 ? 4 : 8;
    constexpr int S = M < C ? M : C;          // entries of one group inside a lane
    constexpr int G = M > C ? M / C : 1;      // lanes per group
    int lo = 0, hi = (int)args.n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (args.d[mid].wg0 <= blockIdx.x)
            lo = mid;
        else
            hi = mid - 1;
    }
    const DenseDev d = args.d[lo];
    const uint32_t total = d.rows * d.chunks_per_row;
    const uint32_t stride = d.n_wg * kThreads;
    constexpr int U = 4;
    for (uint32_t base = (blockIdx.x - d.wg0) * U * kThreads; base < total; base += U * stride) {
        u32x4 raw[U];
        uint32_t keep[U];                       // C keep bits
        size_t out_off[U];
#pragma unroll
        for (int u = 0; u < U; u++) {
            const uint32_t c = base + (uint32_t)u * kThreads + threadIdx.x;
            raw[u] = u32x4{0u, 0u, 0u, 0u};
            keep[u] = 0u;
            out_off[u] = 0;
            if (c < total) {
                const uint32_t r = c / d.chunks_per_row, j = c - r * d.chunks_per_row;
                raw[u] = __builtin_nontemporal_load((const u32x4 *)(d.w + (size_t)r * d.ld_b + (size_t)j * 16u));
                const unsigned char *mrow = d.mask + (size_t)r * d.mask_ld;
                if constexpr (FMT == kMaskU8) {
                    if constexpr (C == 4) {
                        keep[u] = bytes4_to_bits(__builtin_nontemporal_load((const uint32_t *)(mrow + (size_t)j * 4u)));
                    } else {
                        const u32x2 mb = __builtin_nontemporal_load((const u32x2 *)(mrow + (size_t)j * 8u));
                        keep[u] = bytes4_to_bits(mb.x) | (bytes4_to_bits(mb.y) << 4);
                    }
                } else {
                    if constexpr (C == 4)
                        keep[u] = ((uint32_t)mrow[j >> 1] >> ((j & 1u) * 4u)) & 0xFu;
                    else
                        keep[u] = (uint32_t)mrow[j];
                }
                out_off[u] = (size_t)r * d.ld_out_b + (size_t)j * 16u;
            }
        }
#pragma unroll
        for (int u = 0; u < U; u++) {
            float v[C];
            const uint32_t q[4] = {raw[u].x, raw[u].y, raw[u].z, raw[u].w};
            if constexpr (DT == kF32) {
#pragma unroll
                for (int c = 0; c < 4; c++)
                    v[c] = __uint_as_float(q[c]);
            } else {
#pragma unroll
                for (int c = 0; c < 4; c++) {
                    v[2 * c] = __uint_as_float(q[c] << 16);
                    v[2 * c + 1] = __uint_as_float(q[c] & 0xFFFF0000u);
                }
            }
            if constexpr (ABSORB) {
#pragma unroll
                for (int g = 0; g < C / S; g++) {
                    float ps = 0.f;
                    uint32_t pc = 0;
#pragma unroll
                    for (int c = g * S; c < (g + 1) * S; c++) {
                        const bool k = (keep[u] >> c) & 1u;
                        ps += k ? 0.f : v[c];
                        pc += k ? 0u : 1u;
                    }
#pragma unroll
                    for (int o = 1; o < G; o <<= 1) {
                        ps += __shfl_xor(ps, o);
                        pc += (uint32_t)__shfl_xor((int)pc, o);
                    }
                    const float mean = (pc != 0u && pc != (uint32_t)M) ? ps / (float)pc : 0.f;
#pragma unroll
                    for (int c = g * S; c < (g + 1) * S; c++)
                        v[c] = ((keep[u] >> c) & 1u) ? v[c] + mean : 0.f;
                }
            } else {
#pragma unroll
                for (int c = 0; c < C; c++)
                    v[c] = ((keep[u] >> c) & 1u) ? v[c] : 0.f;
            }
            u32x4 o;
            if constexpr (DT == kF32) {
                o = u32x4{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
            } else {
                typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
                typedef float f32x2 __attribute__((ext_vector_type(2)));
                union { bf16x2 h; uint32_t w; } cv[4];
#pragma unroll
                for (int c = 0; c < 4; c++) {
                    if constexpr (ABSORB) {
                        cv[c].h = __builtin_convertvector(f32x2{v[2 * c], v[2 * c + 1]}, bf16x2);   // round to nearest even
                    } else {
                        cv[c].w = (__float_as_uint(v[2 * c]) >> 16) | (__float_as_uint(v[2 * c + 1]) & 0xFFFF0000u);
                    }
                }
                o = u32x4{cv[0].w, cv[1].w, cv[2].w, cv[3].w};
            }
            const uint32_t c = base + (uint32_t)u * kThreads + threadIdx.x;
            if (c < total)
                stream_store(o, (u32x4 *)(d.out + out_off[u]));
        }
    }
}

typedef void (*dense_kernel_t)(const DenseArgs);

template <int DT, int FMT>
static dense_kernel_t pick_dense(int M, bool absorb)
{
    if (!absorb)
        return apply_dense_kernel<DT, FMT, 4, false>;
    switch (M) {
    case 2: return apply_dense_kernel<DT, FMT, 2, true>;
    case 4: return apply_dense_kernel<DT, FMT, 4, true>;
    case 8: return apply_dense_kernel<DT, FMT, 8, true>;
    case 16: return apply_dense_kernel<DT, FMT, 16, true>;
    case 32: return apply_dense_kernel<DT, FMT, 32, true>;
    }
    return nullptr;
}

}  // namespace tmask

namespace tmask {

// Element-wise forms of the masked copy and of the violation count, for matrices that miss the 16-byte alignment of
// the kernels above: a lane takes one entry, a wavefront 64 consecutive columns of a row (a group of M <= 32 columns
// is then an aligned run of lanes: sums by butterfly, counts from the wavefront's ballot).  d.pad = cols,
// d.chunks_per_row = runs of 64 columns per row.  MODE 0: out = W (.) S; 1: the same with the mean of every group's
// pruned weights added to its kept ones; 2: count the non-zero entries the mask removes.
template <int DT, int FMT, int MODE>
__global__ __launch_bounds__(kThreads) void dense_elementwise_kernel(const DenseArgs args, const uint32_t M)
{
    __shared__ uint32_t red[kThreads / 64];
    int lo = 0, hi = (int)args.n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (args.d[mid].wg0 <= blockIdx.x)
            lo = mid;
        else
            hi = mid - 1;
    }
    const DenseDev d = args.d[lo];
    constexpr uint32_t ES = DT == kF32 ? 4u : 2u;
    const uint32_t cols = d.pad, lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t total = d.rows * d.chunks_per_row;
    uint32_t cnt = 0;
    for (uint32_t u = (blockIdx.x - d.wg0) * (kThreads / 64) + wave; u < total; u += d.n_wg * (kThreads / 64)) {
        const uint32_t r = u / d.chunks_per_row, c = (u - r * d.chunks_per_row) * 64u + lane;
        const bool active = c < cols;
        uint32_t raw = 0;
        bool keep = false;
        if (active) {
            const char *src = d.w + (size_t)r * d.ld_b + (size_t)c * ES;
            raw = DT == kF32 ? *(const uint32_t *)src : (uint32_t) * (const uint16_t *)src;
            if constexpr (FMT == kMaskU8)
                keep = d.mask[(size_t)r * d.mask_ld + c] != 0;
            else
                keep = ((d.mask[(size_t)r * d.mask_ld + (c >> 3)] >> (c & 7u)) & 1u) != 0;
        }
        if constexpr (MODE == 2) {
            const uint32_t mag = DT == kF32 ? (raw & 0x7FFFFFFFu) : (raw & 0x7FFFu);
            cnt += (active && mag != 0u && !keep) ? 1u : 0u;
        } else {
            uint32_t o = keep ? raw : 0u;
            if constexpr (MODE == 1) {
                const float v = DT == kF32 ? __uint_as_float(raw) : __uint_as_float(raw << 16);
                float ps = (active && !keep) ? v : 0.f;
                for (uint32_t off = M >> 1; off >= 1u; off >>= 1)
                    ps += __shfl_xor(ps, (int)off, 64);
                const unsigned long long kb = __builtin_amdgcn_ballot_w64(keep);
                const uint32_t seg = (uint32_t)(kb >> (lane & ~(M - 1u))) & (uint32_t)((1ull << M) - 1ull);
                const uint32_t pc = M - (uint32_t)__builtin_popcount(seg);
                const float mean = (pc != 0u && pc != M) ? ps / (float)pc : 0.f;
                const float res = keep ? v + mean : 0.f;
                if constexpr (DT == kF32) {
                    o = __float_as_uint(res);
                } else {
                    const uint32_t b = __float_as_uint(res);
                    o = ((b & 0x7FFFFFFFu) > 0x7F800000u) ? ((b >> 16) | 0x0040u) : ((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16);
                }
            }
            if (active) {
                char *dst = d.out + (size_t)r * d.ld_out_b + (size_t)c * ES;
                if constexpr (DT == kF32)
                    *(uint32_t *)dst = o;
                else
                    *(uint16_t *)dst = (uint16_t)o;
            }
        }
    }
    if constexpr (MODE == 2) {
        const uint32_t t = block_sum(cnt, red);
        if (threadIdx.x == 0 && t)
            atomicAdd((unsigned long long *)d.out, (unsigned long long)t);
    }
}

typedef void (*dense_elementwise_t)(const DenseArgs, const uint32_t);

__global__ void violation_zero_kernel(const DenseArgs args);

template <int MODE>
static dense_elementwise_t pick_elementwise(int dt, int mf)
{
    return dt == TMASK_F32 ? (mf == TMASK_MASK_U8 ? dense_elementwise_kernel<kF32, kMaskU8, MODE> : dense_elementwise_kernel<kF32, kMaskBits, MODE>)
                           : (mf == TMASK_MASK_U8 ? dense_elementwise_kernel<kBF16, kMaskU8, MODE> : dense_elementwise_kernel<kBF16, kMaskBits, MODE>);
}

// launches the element-wise kernel over descriptors already filled except for the work split
static int launch_elementwise(dense_elementwise_t kern, DenseArgs &args, int nb, uint32_t M, bool zero_first, hipStream_t stream,
                              bool last)
{
    uint32_t wgs = 0;
    for (int k = 0; k < nb; k++) {
        DenseDev &d = args.d[k];
        const uint64_t units = (uint64_t)d.rows * d.chunks_per_row;
        uint64_t nw = (units + 15) / 16;                    // four wavefronts per workgroup, four runs each
        nw = nw < 1 ? 1 : nw > 4096 ? 4096 : nw;
        d.n_wg = (uint32_t)nw; d.wg0 = wgs;
        wgs += d.n_wg;
    }
    args.n = (uint32_t)nb;
    if (zero_first)
        hipLaunchKernelGGL(violation_zero_kernel, dim3(1), dim3(kMaxDenseBatch), 0, stream, args);
    {
        ProfileScope prof(stream, last);
        hipLaunchKernelGGL(kern, dim3(wgs), dim3(kThreads), 0, stream, args, M);
    }
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? TMASK_OK : hip_fail(e, "element-wise masked copy / count launch");
}

}  // namespace tmask

extern "C" int tmask_apply_dense(const tmask_dense_desc *descs, int n, tmask_dtype dt, int M, int absorb_mean,
                                 tmask_mask_fmt mf, void *hip_stream)
{
    if (!descs)
        return fail(TMASK_ERR_NULL, "descriptor array is NULL");
    if (n <= 0)
        return fail(TMASK_ERR_SHAPE, "n=%d must be positive", n);
    if (dt != TMASK_F32 && dt != TMASK_BF16)
        return fail(TMASK_ERR_DTYPE, "unknown dtype %d", (int)dt);
    if (mf != TMASK_MASK_U8 && mf != TMASK_MASK_BITS)
        return fail(TMASK_ERR_DTYPE, "unknown mask format %d", (int)mf);
    if (absorb_mean && M != 2 && M != 4 && M != 8 && M != 16 && M != 32)
        return fail(TMASK_ERR_NM, "mean absorption needs M in {2, 4, 8, 16, 32} (M=%d)", M);
    const int64_t es = dt == TMASK_F32 ? 4 : 2, per_chunk = 16 / es;
    bool aligned = true;
    for (int i = 0; i < n; i++) {
        const tmask_dense_desc &f = descs[i];
        if (!f.w || !f.mask || !f.out)
            return fail(TMASK_ERR_NULL, "matrix %d: w, mask or out is NULL", i);
        if (f.rows <= 0 || f.cols <= 0 || (absorb_mean && f.cols % M) || (mf == TMASK_MASK_BITS && f.cols % 8))
            return fail(TMASK_ERR_SHAPE, "matrix %d: rows=%lld cols=%lld (cols must be positive%s%s)", i,
                        (long long)f.rows, (long long)f.cols, absorb_mean ? ", a multiple of M" : "",
                        mf == TMASK_MASK_BITS ? ", a multiple of 8 for BITS masks" : "");
        const int64_t mask_row = mf == TMASK_MASK_U8 ? f.cols : f.cols / 8;
        if (f.ld < f.cols || f.ld_out < f.cols || f.mask_ld < mask_row || f.ld * es > 0x7FFFFFFFll ||
            f.ld_out * es > 0x7FFFFFFFll || f.mask_ld > 0x7FFFFFFFll || f.rows * ((f.cols + per_chunk - 1) / per_chunk) >= 0xFFFFFFFFll)
            return fail(TMASK_ERR_SHAPE, "matrix %d: leading dimensions must cover a row; at most 2^32 - 1 chunks of 16 bytes",
                        i);
        if (((uintptr_t)f.w | (uintptr_t)f.out) % (uintptr_t)es)
            return fail(TMASK_ERR_ALIGN, "matrix %d: w and out must be aligned to the element size", i);
        if ((((uintptr_t)f.w | (uintptr_t)f.out | (uint64_t)(f.ld * es) | (uint64_t)(f.ld_out * es)) & 15) || f.cols % per_chunk)
            aligned = false;
        if (mf == TMASK_MASK_U8 && (((uintptr_t)f.mask | (uint64_t)f.mask_ld) & (uint64_t)(per_chunk - 1)))
            aligned = false;
    }
    const bool absorb = absorb_mean != 0;
    if (!aligned) {      // element-wise kernel: any layout
        const dense_elementwise_t ek = absorb ? pick_elementwise<1>((int)dt, (int)mf) : pick_elementwise<0>((int)dt, (int)mf);
        for (int first = 0; first < n; first += kMaxDenseBatch) {
            const int nb = n - first < kMaxDenseBatch ? n - first : kMaxDenseBatch;
            DenseArgs args;
            memset(&args, 0, sizeof args);
            for (int k = 0; k < nb; k++) {
                const tmask_dense_desc &f = descs[first + k];
                DenseDev &d = args.d[k];
                d.w = (const char *)f.w; d.mask = (const unsigned char *)f.mask; d.out = (char *)f.out;
                d.rows = (uint32_t)f.rows; d.chunks_per_row = (uint32_t)((f.cols + 63) / 64); d.pad = (uint32_t)f.cols;
                d.ld_b = (uint32_t)(f.ld * es); d.ld_out_b = (uint32_t)(f.ld_out * es); d.mask_ld = (uint32_t)f.mask_ld;
            }
            const int rc = launch_elementwise(ek, args, nb, (uint32_t)(absorb ? M : 1), false, (hipStream_t)hip_stream,
                                              first + kMaxDenseBatch >= n);
            if (rc)
                return rc;
        }
        return TMASK_OK;
    }
    dense_kernel_t kern = dt == TMASK_F32 ? (mf == TMASK_MASK_U8 ? pick_dense<kF32, kMaskU8>(M, absorb)
                                                                 : pick_dense<kF32, kMaskBits>(M, absorb))
                                          : (mf == TMASK_MASK_U8 ? pick_dense<kBF16, kMaskU8>(M, absorb)
                                                                 : pick_dense<kBF16, kMaskBits>(M, absorb));
    hipStream_t stream = (hipStream_t)hip_stream;
    for (int first = 0; first < n; first += kMaxDenseBatch) {
        const int nb = n - first < kMaxDenseBatch ? n - first : kMaxDenseBatch;
        DenseArgs args;
        memset(&args, 0, sizeof args);
        uint32_t wgs = 0;
        for (int k = 0; k < nb; k++) {
            const tmask_dense_desc &f = descs[first + k];
            DenseDev &d = args.d[k];
            d.w = (const char *)f.w; d.mask = (const unsigned char *)f.mask; d.out = (char *)f.out;
            d.rows = (uint32_t)f.rows; d.chunks_per_row = (uint32_t)(f.cols / per_chunk);
            d.ld_b = (uint32_t)(f.ld * es); d.ld_out_b = (uint32_t)(f.ld_out * es); d.mask_ld = (uint32_t)f.mask_ld;
            const uint64_t chunks = (uint64_t)d.rows * d.chunks_per_row;
            uint64_t nw = (chunks + 4ull * kThreads - 1) / (4ull * kThreads);
            nw = nw < 1 ? 1 : nw > 8192 ? 8192 : nw;
            d.n_wg = (uint32_t)nw; d.wg0 = wgs;
            wgs += d.n_wg;
        }
        args.n = (uint32_t)nb;
        {
            ProfileScope prof(stream, first + kMaxDenseBatch >= n);
            hipLaunchKernelGGL(kern, dim3(wgs), dim3(kThreads), 0, stream, args);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return hip_fail(e, "apply_dense launch");
    }
    return TMASK_OK;
}

// ---------------------------------------------------------------------------------------------------------
// Pattern violations (Sec. 5): non-zero weights that a mask removes.  Streams W and the mask like the dense copy
// (DenseDev with `out` = the matrix' counter), counts with integer atomics like the flip counter.
// ---------------------------------------------------------------------------------------------------------
namespace tmask {

__global__ void violation_zero_kernel(const DenseArgs args)
{
    if (threadIdx.x < args.n)
        *(unsigned long long *)args.d[threadIdx.x].out = 0ull;
}

template <int DT, int FMT>
__global__ __launch_bounds__(kThreads) void violation_count_kernel(const DenseArgs args)
{
    constexpr int C = DT == kF32 ? 4 : 8;
    __shared__ uint32_t red[kThreads / 64];
    int lo = 0, hi = (int)args.n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (args.d[mid].wg0 <= blockIdx.x)
            lo = mid;
        else
            hi = mid - 1;
    }
    const DenseDev d = args.d[lo];
    const uint32_t total = d.rows * d.chunks_per_row;
    const uint32_t stride = d.n_wg * kThreads;
    uint32_t cnt = 0;
    constexpr int U = 4;
    for (uint32_t base = (blockIdx.x - d.wg0) * U * kThreads; base < total; base += U * stride) {
        u32x4 raw[U];
        uint32_t keep[U];
#pragma unroll
        for (int u = 0; u < U; u++) {
            const uint32_t c = base + (uint32_t)u * kThreads + threadIdx.x;
            raw[u] = u32x4{0u, 0u, 0u, 0u};
            keep[u] = 0u;
            if (c < total) {
                const uint32_t r = c / d.chunks_per_row, j = c - r * d.chunks_per_row;
                raw[u] = __builtin_nontemporal_load((const u32x4 *)(d.w + (size_t)r * d.ld_b + (size_t)j * 16u));
                const unsigned char *mrow = d.mask + (size_t)r * d.mask_ld;
                if constexpr (FMT == kMaskU8) {
                    if constexpr (C == 4) {
                        keep[u] = bytes4_to_bits(__builtin_nontemporal_load((const uint32_t *)(mrow + (size_t)j * 4u)));
                    } else {
                        const u32x2 mb = __builtin_nontemporal_load((const u32x2 *)(mrow + (size_t)j * 8u));
                        keep[u] = bytes4_to_bits(mb.x) | (bytes4_to_bits(mb.y) << 4);
                    }
                } else {
                    if constexpr (C == 4)
                        keep[u] = ((uint32_t)mrow[j >> 1] >> ((j & 1u) * 4u)) & 0xFu;
                    else
                        keep[u] = (uint32_t)mrow[j];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; u++) {
            const uint32_t q[4] = {raw[u].x, raw[u].y, raw[u].z, raw[u].w};
            uint32_t active = 0;                         // bit c = entry c is not +-0
#pragma unroll
            for (int c = 0; c < 4; c++) {
                if constexpr (DT == kF32) {
                    active |= ((q[c] & 0x7FFFFFFFu) != 0u ? 1u : 0u) << c;
                } else {
                    active |= ((q[c] & 0x00007FFFu) != 0u ? 1u : 0u) << (2 * c);
                    active |= ((q[c] & 0x7FFF0000u) != 0u ? 1u : 0u) << (2 * c + 1);
                }
            }
            cnt += (uint32_t)__builtin_popcount(active & ~keep[u]);      // lanes past the end hold zeros: nothing active
        }
    }
    const uint32_t t = block_sum(cnt, red);
    if (threadIdx.x == 0 && t)
        atomicAdd((unsigned long long *)d.out, (unsigned long long)t);   // integer sum: order does not matter
}

}  // namespace tmask

extern "C" int tmask_pattern_violations(const tmask_violation_desc *descs, int n, tmask_dtype dt, tmask_mask_fmt mf,
                                        void *hip_stream)
{
    if (!descs)
        return fail(TMASK_ERR_NULL, "descriptor array is NULL");
    if (n <= 0)
        return fail(TMASK_ERR_SHAPE, "n=%d must be positive", n);
    if (dt != TMASK_F32 && dt != TMASK_BF16)
        return fail(TMASK_ERR_DTYPE, "unknown dtype %d", (int)dt);
    if (mf != TMASK_MASK_U8 && mf != TMASK_MASK_BITS)
        return fail(TMASK_ERR_DTYPE, "unknown mask format %d", (int)mf);
    const int64_t es = dt == TMASK_F32 ? 4 : 2, per_chunk = 16 / es;
    bool aligned = true;
    for (int i = 0; i < n; i++) {
        const tmask_violation_desc &f = descs[i];
        if (!f.w || !f.mask || !f.count)
            return fail(TMASK_ERR_NULL, "matrix %d: w, mask or count is NULL", i);
        if (f.rows <= 0 || f.cols <= 0 || (mf == TMASK_MASK_BITS && f.cols % 8))
            return fail(TMASK_ERR_SHAPE, "matrix %d: rows=%lld cols=%lld (cols must be positive%s)", i,
                        (long long)f.rows, (long long)f.cols, mf == TMASK_MASK_BITS ? ", a multiple of 8 for BITS masks" : "");
        const int64_t mask_row = mf == TMASK_MASK_U8 ? f.cols : f.cols / 8;
        if (f.ld < f.cols || f.mask_ld < mask_row || f.ld * es > 0x7FFFFFFFll || f.mask_ld > 0x7FFFFFFFll ||
            f.rows * ((f.cols + per_chunk - 1) / per_chunk) >= 0xFFFFFFFFll)
            return fail(TMASK_ERR_SHAPE, "matrix %d: leading dimensions must cover a row; at most 2^32 - 1 chunks of 16 bytes", i);
        if ((uintptr_t)f.w % (uintptr_t)es)
            return fail(TMASK_ERR_ALIGN, "matrix %d: w must be aligned to the element size", i);
        if ((((uintptr_t)f.w | (uint64_t)(f.ld * es)) & 15) || f.cols % per_chunk)
            aligned = false;
        if (mf == TMASK_MASK_U8 && (((uintptr_t)f.mask | (uint64_t)f.mask_ld) & (uint64_t)(per_chunk - 1)))
            aligned = false;
        if ((uintptr_t)f.count & 7)
            return fail(TMASK_ERR_ALIGN, "matrix %d: count must be 8-byte aligned", i);
    }
    if (!aligned) {      // element-wise kernel: any layout
        const dense_elementwise_t ek = pick_elementwise<2>((int)dt, (int)mf);
        for (int first = 0; first < n; first += kMaxDenseBatch) {
            const int nb = n - first < kMaxDenseBatch ? n - first : kMaxDenseBatch;
            DenseArgs args;
            memset(&args, 0, sizeof args);
            for (int k = 0; k < nb; k++) {
                const tmask_violation_desc &f = descs[first + k];
                DenseDev &d = args.d[k];
                d.w = (const char *)f.w; d.mask = (const unsigned char *)f.mask; d.out = (char *)f.count;
                d.rows = (uint32_t)f.rows; d.chunks_per_row = (uint32_t)((f.cols + 63) / 64); d.pad = (uint32_t)f.cols;
                d.ld_b = (uint32_t)(f.ld * es); d.ld_out_b = 0; d.mask_ld = (uint32_t)f.mask_ld;
            }
            const int rc = launch_elementwise(ek, args, nb, 1u, true, (hipStream_t)hip_stream, first + kMaxDenseBatch >= n);
            if (rc)
                return rc;
        }
        return TMASK_OK;
    }
    dense_kernel_t kern = dt == TMASK_F32 ? (mf == TMASK_MASK_U8 ? violation_count_kernel<kF32, kMaskU8>
                                                                 : violation_count_kernel<kF32, kMaskBits>)
                                          : (mf == TMASK_MASK_U8 ? violation_count_kernel<kBF16, kMaskU8>
                                                                 : violation_count_kernel<kBF16, kMaskBits>);
    hipStream_t stream = (hipStream_t)hip_stream;
    for (int first = 0; first < n; first += kMaxDenseBatch) {
        const int nb = n - first < kMaxDenseBatch ? n - first : kMaxDenseBatch;
        DenseArgs args;
        memset(&args, 0, sizeof args);
        uint32_t wgs = 0;
        for (int k = 0; k < nb; k++) {
            const tmask_violation_desc &f = descs[first + k];
            DenseDev &d = args.d[k];
            d.w = (const char *)f.w; d.mask = (const unsigned char *)f.mask; d.out = (char *)f.count;
            d.rows = (uint32_t)f.rows; d.chunks_per_row = (uint32_t)(f.cols / per_chunk);
            d.ld_b = (uint32_t)(f.ld * es); d.ld_out_b = 0; d.mask_ld = (uint32_t)f.mask_ld;
            const uint64_t chunks = (uint64_t)d.rows * d.chunks_per_row;
            uint64_t nw = (chunks + 4ull * kThreads - 1) / (4ull * kThreads);
            nw = nw < 1 ? 1 : nw > 1024 ? 1024 : nw;       // one atomic per workgroup: keep them few, as in the flip counter
            d.n_wg = (uint32_t)nw; d.wg0 = wgs;
            wgs += d.n_wg;
        }
        args.n = (uint32_t)nb;
        hipLaunchKernelGGL(violation_zero_kernel, dim3(1), dim3(kMaxDenseBatch), 0, stream, args);
        {
            ProfileScope prof(stream, first + kMaxDenseBatch >= n);
            hipLaunchKernelGGL(kern, dim3(wgs), dim3(kThreads), 0, stream, args);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return hip_fail(e, "pattern violation count launch");
    }
    return TMASK_OK;
}

// log10 of the number of masks a constraint admits on a tensor of T elements at sparsity N/M (Eq. 2).
extern "C" int tmask_mask_diversity(tmask_md_kind kind, int N, int M, int64_t T, double *log10_md)
{
    if (!log10_md)
        return fail(TMASK_ERR_NULL, "log10_md is NULL");
    if (M < 2 || N <= 0 || N >= M || T <= 0)
        return fail(TMASK_ERR_NM, "need 0 < N < M and T > 0 (N=%d M=%d T=%lld)", N, M, (long long)T);
    const double ln10 = std::log(10.0);
    auto lfact = [](double v) { return std::lgamma(v + 1.0); };
    double ln = 0.0;
    switch (kind) {
    case TMASK_MD_UNSTRUCTURED: {
        if ((T * N) % M)
            return fail(TMASK_ERR_SHAPE, "T*N must be a multiple of M");
        const double k = (double)(T * N / M);
        ln = lfact((double)T) - lfact(k) - lfact((double)T - k);
        break;
    }
    case TMASK_MD_STRUCTURED:
        if (T % M)
            return fail(TMASK_ERR_SHAPE, "T must be a multiple of M");
        ln = (double)(T / M) * (lfact(M) - lfact(N) - lfact(M - N));
        break;
    case TMASK_MD_TRANSPOSABLE: {
        if (T % ((int64_t)M * M))
            return fail(TMASK_ERR_SHAPE, "T must be a multiple of M*M");
        double per_block = 0.0;
        for (int q = 0; q < N; q++)
            per_block += lfact(M - q);                 // M! (M-1)! ... (M-N+1)!
        ln = (double)(T / ((int64_t)M * M)) * per_block;
        break;
    }
    case TMASK_MD_SEQUENTIAL:
        if (T % M)
            return fail(TMASK_ERR_SHAPE, "T must be a multiple of M");
        ln = (double)(T / M) * std::log((double)(M - N + 1));
        break;
    default:
        return fail(TMASK_ERR_DTYPE, "unknown constraint kind %d", (int)kind);
    }
    *log10_md = ln / ln10;
    return TMASK_OK;
}

// Probability that a block of M i.i.d. entries, each prunable with probability rho, has at least N prunable
// ones (Sec. 5, Eq. 4): the upper tail of the binomial distribution.
extern "C" int tmask_nm_sparse_probability(int N, int M, double rho, double *prob)
{
    if (!prob)
        return fail(TMASK_ERR_NULL, "prob is NULL");
    if (M < 1 || M > 1024 || N < 0 || N > M || !(rho >= 0.0 && rho <= 1.0))
        return fail(TMASK_ERR_NM, "need 0 <= N <= M <= 1024 and 0 <= rho <= 1 (N=%d M=%d rho=%g)", N, M, rho);
    double sum = 0.0;
    for (int i = N; i <= M; i++) {
        // C(M, i) rho^i (1 - rho)^(M - i), in logs to stay in range; the end points 0 and 1 need no logs
        double term;
        if (rho == 0.0)
            term = i == 0 ? 1.0 : 0.0;
        else if (rho == 1.0)
            term = i == M ? 1.0 : 0.0;
        else
            term = std::exp(std::lgamma(M + 1.0) - std::lgamma(i + 1.0) - std::lgamma(M - i + 1.0) + i * std::log(rho) +
                            (M - i) * std::log1p(-rho));
        sum += term;
    }
    *prob = sum > 1.0 ? 1.0 : sum;
    return TMASK_OK;
}

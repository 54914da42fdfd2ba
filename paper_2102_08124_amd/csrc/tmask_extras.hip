// Small companions of the mask kernels: the mask-flip counter of a dynamic-mask training loop and the
// mask-diversity formulas (arXiv 2102.08124, Sec. 3, Eq. 2) with the N:M probability of Sec. 5, Eq. 4.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstring>

#include "../../include/tmask.h"
#include "tmask_device.hpp"
#include "tmask_host.hpp"

namespace tmask {

constexpr int kMaxFlipBatch = 64;

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
static_assert(sizeof(FlipArgs) <= 4096, "descriptor table must fit the kernel-argument segment");

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

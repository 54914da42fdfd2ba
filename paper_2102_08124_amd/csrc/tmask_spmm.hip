// tmask_spmm24: products with the compressed 2:4 operands written by tmask_apply_pack / tmask_approx_pack,
// on the structured-sparse matrix cores of gfx950 (arXiv 2102.08124, Sec. 1, Eq. 1, and Sec. 4: the forward
// product uses W, the backward product W^T, and a transposable mask makes both of them 2:4 sparse).
//
//     y[t][r] = sum_c x[t][c] * Wd[r][c],   Wd = the rows x cols matrix whose compressed form is (vals, idx)
//
// The instruction: D(16x16, fp32) += A(16x64, 2:4 sparse along k, bf16) * B(64x16, bf16).  Lane l of the
// wavefront holds, with m = l % 16 and a = l / 16:
//   A: 8 compressed values of row m: the two values of each of the groups of four g0, g0+1, g0+4, g0+5,
//      g0 = 8 (a % 2) + 2 (a / 2), i.e. two runs of four consecutive compressed values;
//   index register: bits 2j..2j+1 = position inside its group of the j-th value, j = 0..7 (low 16 bits);
//   B: 16 consecutive k of column n = m: k = 16 a .. 16 a + 15;
//   D: rows 4 a .. 4 a + 3 of column m.
// (Layout established by one-hot probes on the hardware; the tests compare whole products with a CPU
// reference, which fixes every part of it.)  One byte of the packed `idx` array holds the positions of
// two consecutive groups, low nibble first, two bits per value in slot order: exactly eight index bits of
// the instruction, so the packed operands feed it unchanged.
//
// Tiling: a workgroup (4 wavefronts, 2 x 2) computes 128 rows x 128 tokens; each wavefront 64 x 64 =
// 4 x 4 instruction tiles (64 accumulator registers).  k advances by 64 per step; the compressed A tile
// (128 x 32 values + 128 x 8 index bytes) and the B tile (128 tokens x 64) go global -> registers -> LDS,
// double-buffered, one barrier per step.  LDS rows are padded so that fragment reads are conflict-free.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/tmask.h"
#include "tmask_host.hpp"

namespace tmask {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t su32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t su32x2 __attribute__((ext_vector_type(2)));

constexpr int kSpThreads = 256;
constexpr int kSpTR = 128;          // rows of Wd per workgroup
constexpr int kSpTT = 128;          // tokens per workgroup
constexpr int kSpKS = 64;           // k per step (one instruction deep)
constexpr int kSpAPitch = 72;       // bytes per LDS row of compressed A (64 data + 8 pad)
constexpr int kSpBPitch = 144;      // bytes per LDS row of B (128 data + 16 pad)
constexpr int kSpIPitch = 8;        // index bytes per row and step

struct SpmmArgs {
    const void *vals;     // rows x cols/2 bf16
    const void *idx;      // rows x cols/8 bytes
    const void *x;        // tokens x cols bf16, leading dimension ld_x
    void *y;              // tokens x rows, leading dimension ld_y
    uint32_t rows, cols, tokens;
    uint32_t ld_x, ld_y;
    uint32_t tiles_r, tiles_t;
};

template <bool OUT_BF16>
__global__ __launch_bounds__(kSpThreads) void spmm24_kernel(const SpmmArgs p)
{
    __shared__ __attribute__((aligned(16))) unsigned char As[2][kSpTR * kSpAPitch];
    __shared__ __attribute__((aligned(16))) unsigned char Bs[2][kSpTT * kSpBPitch];
    __shared__ __attribute__((aligned(16))) unsigned char Is[2][kSpTR * kSpIPitch];

    // Workgroups are handed to the eight XCDs round-robin; give each XCD a contiguous range of tiles so
    // that the tiles sharing rows of Wd meet in one L2.
    const uint32_t n_tiles = p.tiles_r * p.tiles_t;
    uint32_t id = blockIdx.x;
    {
        const uint32_t per = n_tiles / 8u;
        if (id < per * 8u)
            id = (id & 7u) * per + (id >> 3);
    }
    const uint32_t tr = id / p.tiles_t, tt = id - tr * p.tiles_t;
    const uint32_t row0 = tr * kSpTR, tok0 = tt * kSpTT;
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t wr = wave >> 1, wc = wave & 1u;

    // ---- global -> register staging (rows and tokens past the edge re-read the last valid one) ----
    const uint32_t g_row = min(row0 + (tid >> 1), p.rows - 1u);       // A: 2 threads per row, 32 B each
    const uint32_t g_tok = min(tok0 + (tid >> 1), p.tokens - 1u);     // B: 2 threads per token, 64 B each
    const uint32_t i_row = min(row0 + (tid & 127u), p.rows - 1u);     // idx: threads 0..127, 8 B each
    const unsigned char *ga = (const unsigned char *)p.vals + (size_t)g_row * p.cols + (tid & 1u) * 32u;
    const unsigned char *gb = (const unsigned char *)p.x + (size_t)g_tok * p.ld_x * 2u + (tid & 1u) * 64u;
    const unsigned char *gi = (const unsigned char *)p.idx + (size_t)i_row * (p.cols >> 3);
    su32x4 ra[2], rb[4];
    su32x2 ri = {0u, 0u};
    auto fetch = [&](uint32_t k0) {
        // compressed A: cols/2 values per row = cols bytes per row; a step covers 32 values = 64 bytes
        ra[0] = *(const su32x4 *)(ga + (size_t)k0);
        ra[1] = *(const su32x4 *)(ga + (size_t)k0 + 16);
#pragma unroll
        for (int i = 0; i < 4; i++)
            rb[i] = *(const su32x4 *)(gb + (size_t)k0 * 2u + 16 * i);
        if (tid < 128u)
            ri = *(const su32x2 *)(gi + (k0 >> 3));
    };
    auto stash = [&](int buf) {
        unsigned char *da = &As[buf][(tid >> 1) * kSpAPitch + (tid & 1u) * 32u];
        *(su32x2 *)(da) = su32x2{ra[0].x, ra[0].y};          // rows are 8-byte aligned only (pitch 72)
        *(su32x2 *)(da + 8) = su32x2{ra[0].z, ra[0].w};
        *(su32x2 *)(da + 16) = su32x2{ra[1].x, ra[1].y};
        *(su32x2 *)(da + 24) = su32x2{ra[1].z, ra[1].w};
        unsigned char *db = &Bs[buf][(tid >> 1) * kSpBPitch + (tid & 1u) * 64u];
#pragma unroll
        for (int i = 0; i < 4; i++)
            *(su32x4 *)(db + 16 * i) = rb[i];
        if (tid < 128u)
            *(su32x2 *)&Is[buf][tid * kSpIPitch] = ri;
    };

    f32x4 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++)
            acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    const uint32_t m = lane & 15u, a = lane >> 4;
    // the lane's two runs of compressed A inside a step: groups g0, g0+1 (8 bytes) and g0+4, g0+5
    const uint32_t g0 = 8u * (a & 1u) + 2u * (a >> 1);
    const uint32_t a_off = g0 * 4u;                 // bytes: 2 values x 2 bytes per group
    const uint32_t i_off = g0 >> 1;                 // index byte of groups g0, g0+1; groups g0+4, g0+5 are 2 further

    const uint32_t steps = p.cols / kSpKS;
    fetch(0);
    stash(0);
    __syncthreads();
    for (uint32_t s = 0; s < steps; s++) {
        const int cur = (int)(s & 1u);
        if (s + 1 < steps)
            fetch((s + 1) * kSpKS);
        // B fragments of the wavefront's four token tiles
        bf16x16 bfrag[4];
#pragma unroll
        for (int ct = 0; ct < 4; ct++) {
            const unsigned char *src = &Bs[cur][(wc * 64u + ct * 16u + m) * kSpBPitch + a * 32u];
            union { su32x4 u[2]; bf16x16 v; } cv;
            cv.u[0] = *(const su32x4 *)src;
            cv.u[1] = *(const su32x4 *)(src + 16);
            bfrag[ct] = cv.v;
        }
#pragma unroll
        for (int rt = 0; rt < 4; rt++) {
            const uint32_t r = wr * 64u + rt * 16u + m;
            const unsigned char *src = &As[cur][r * kSpAPitch + a_off];
            union { su32x2 u[2]; bf16x8 v; } av;
            av.u[0] = *(const su32x2 *)src;
            av.u[1] = *(const su32x2 *)(src + 16);
            const unsigned char *is = &Is[cur][r * kSpIPitch + i_off];
            const int sel = (int)((uint32_t)is[0] | ((uint32_t)is[2] << 8));
#pragma unroll
            for (int ct = 0; ct < 4; ct++)
                acc[rt][ct] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(av.v, bfrag[ct], acc[rt][ct], sel, 0, 0);
        }
        if (s + 1 < steps)
            stash(cur ^ 1);
        __syncthreads();
    }

    // ---- store: lane holds rows 4a..4a+3 of token column m of each tile: 4 consecutive y entries ----
#pragma unroll
    for (int rt = 0; rt < 4; rt++) {
#pragma unroll
        for (int ct = 0; ct < 4; ct++) {
            const uint32_t tok = tok0 + wc * 64u + ct * 16u + m;
            const uint32_t r = row0 + wr * 64u + rt * 16u + a * 4u;
            if (tok < p.tokens && r < p.rows) {       // rows is a multiple of 4: the four entries are in or out together
                const f32x4 v = acc[rt][ct];
                if constexpr (OUT_BF16) {
                    su32x2 o;
                    auto rne = [](float f) -> uint32_t {
                        const uint32_t u = __float_as_uint(f);
                        if ((u & 0x7FFFFFFFu) > 0x7F800000u)
                            return (u >> 16) | 0x40u;                     // NaN stays NaN
                        return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;    // round to nearest even
                    };
                    o.x = rne(v.x) | (rne(v.y) << 16);
                    o.y = rne(v.z) | (rne(v.w) << 16);
                    *(su32x2 *)((unsigned char *)p.y + ((size_t)tok * p.ld_y + r) * 2u) = o;
                } else {
                    *(f32x4 *)((unsigned char *)p.y + ((size_t)tok * p.ld_y + r) * 4u) = v;
                }
            }
        }
    }
}

}  // namespace tmask

using namespace tmask;

extern "C" int tmask_spmm24(const void *vals, const void *idx, int64_t rows, int64_t cols, const void *x, int64_t ld_x,
                            void *y, int64_t ld_y, int64_t tokens, tmask_dtype out_dt, void *hip_stream)
{
    if (!vals || !idx || !x || !y)
        return fail(TMASK_ERR_NULL, "vals, idx, x or y is NULL");
    if (out_dt != TMASK_F32 && out_dt != TMASK_BF16)
        return fail(TMASK_ERR_DTYPE, "unknown output dtype %d", (int)out_dt);
    if (rows <= 0 || cols <= 0 || tokens <= 0 || rows % 4 || cols % kSpKS || ld_x < cols || ld_y < rows)
        return fail(TMASK_ERR_SHAPE,
                    "rows=%lld (multiple of 4) cols=%lld (multiple of 64) tokens=%lld ld_x=%lld (>= cols) ld_y=%lld (>= rows)",
                    (long long)rows, (long long)cols, (long long)tokens, (long long)ld_x, (long long)ld_y);
    if (rows > 0x7FFFFFFFll || cols > 0x7FFFFFFFll || tokens > 0x7FFFFFFFll || ld_x > 0x7FFFFFFFll || ld_y > 0x7FFFFFFFll)
        return fail(TMASK_ERR_SHAPE, "sizes must stay below 2^31");
    const int64_t ysz = out_dt == TMASK_F32 ? 4 : 2;
    if (((uintptr_t)vals & 15) || ((uintptr_t)idx & 7) || ((uintptr_t)x & 15) || (ld_x % 8) || ((uintptr_t)y & 15) ||
        (ld_y * ysz) % 16)
        return fail(TMASK_ERR_ALIGN,
                    "vals, x, y must be 16-byte aligned, idx 8-byte aligned, ld_x a multiple of 8, ld_y*sizeof(y) a multiple of 16");
    SpmmArgs p;
    p.vals = vals; p.idx = idx; p.x = x; p.y = y;
    p.rows = (uint32_t)rows; p.cols = (uint32_t)cols; p.tokens = (uint32_t)tokens;
    p.ld_x = (uint32_t)ld_x; p.ld_y = (uint32_t)ld_y;
    p.tiles_r = (uint32_t)((rows + kSpTR - 1) / kSpTR);
    p.tiles_t = (uint32_t)((tokens + kSpTT - 1) / kSpTT);
    const uint64_t n_tiles = (uint64_t)p.tiles_r * p.tiles_t;
    if (n_tiles > 0x7FFFFFFFull)
        return fail(TMASK_ERR_SHAPE, "too many tiles");
    hipStream_t stream = (hipStream_t)hip_stream;
    {
        ProfileScope prof(stream, true);
        if (out_dt == TMASK_BF16)
            hipLaunchKernelGGL(spmm24_kernel<true>, dim3((uint32_t)n_tiles), dim3(kSpThreads), 0, stream, p);
        else
            hipLaunchKernelGGL(spmm24_kernel<false>, dim3((uint32_t)n_tiles), dim3(kSpThreads), 0, stream, p);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return hip_fail(e, "spmm kernel launch");
    return TMASK_OK;
}

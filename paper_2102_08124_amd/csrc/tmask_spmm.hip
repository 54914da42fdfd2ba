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
// Tiling: a workgroup (4 wavefronts, 2 x 2) computes 256 rows x 128 tokens; each wavefront 128 x 64 =
// 8 x 4 instruction tiles (128 accumulator registers).  k advances by 64 per step; the compressed A tile
// (256 x 32 values + 256 x 8 index bytes) and the B tile (128 tokens x 64) go global -> registers -> LDS:
// one register set and two LDS buffers, loads run one step ahead of the multiplication; one barrier per
// step.  LDS rows are padded so that fragment reads are conflict-free.
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
constexpr int kSpRT = 8;            // 16-row instruction tiles per wavefront
constexpr int kSpCT = 4;            // 16-token instruction tiles per wavefront
constexpr int kSpTR = 2 * kSpRT * 16;   // rows of Wd per workgroup (2 x 2 wavefronts)
constexpr int kSpTT = 2 * kSpCT * 16;   // tokens per workgroup
constexpr int kSpAL = kSpTR / 64;   // 16-byte pieces of A a thread moves per step
constexpr int kSpBL = kSpTT / 32;   // 16-byte pieces of B a thread moves per step
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
__global__ __launch_bounds__(kSpThreads, 2) void spmm24_kernel(const SpmmArgs p)
{
    __shared__ __attribute__((aligned(16))) unsigned char As[2][kSpTR * kSpAPitch];
    __shared__ __attribute__((aligned(16))) unsigned char Bs[2][kSpTT * kSpBPitch];
    __shared__ __attribute__((aligned(16))) unsigned char Is[2][kSpTR * kSpIPitch];

    // Workgroups are handed to the eight XCDs round-robin; give each XCD a contiguous range of tile numbers,
    // and number the tiles so that 64 consecutive ones form an 8 x 8 block of the output: the workgroups
    // that run on one XCD at the same time then share 8 row panels of Wd and 8 token panels of x in its L2
    // instead of streaming 64 of each.
    const uint32_t n_tiles = p.tiles_r * p.tiles_t;
    uint32_t id = blockIdx.x;
    {
        const uint32_t per = n_tiles / 8u;
        if (id < per * 8u)
            id = (id & 7u) * per + (id >> 3);
    }
    constexpr uint32_t kGroup = 8;
    const uint32_t in_group = kGroup * p.tiles_t;
    const uint32_t group = id / in_group, rem = id - group * in_group;
    const uint32_t first_r = group * kGroup;
    const uint32_t group_rows = min(p.tiles_r - first_r, kGroup);
    const uint32_t tt = rem / group_rows;
    const uint32_t tr = first_r + (rem - tt * group_rows);
    const uint32_t row0 = tr * kSpTR, tok0 = tt * kSpTT;
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t wr = wave >> 1, wc = wave & 1u;

    // ---- global -> register staging (rows and tokens past the edge re-read the last valid one) ----
    // Consecutive lanes fetch consecutive 16-byte pieces of one row, so every load instruction covers whole
    // runs: 8 lanes = the 128 bytes a token contributes to a step, 4 lanes = the 64 bytes of a row of
    // compressed A.  (One lane per row with several pieces each touches four times as many cache lines per
    // instruction and measured twice as slow overall.)
    // Addresses are a wavefront-uniform base (scalar registers) plus a 32-bit lane offset.
    const unsigned char *base_a = (const unsigned char *)p.vals + (size_t)row0 * p.cols;
    const unsigned char *base_b = (const unsigned char *)p.x + (size_t)tok0 * p.ld_x * 2u;
    uint32_t off_b[kSpBL], off_a[kSpAL];
#pragma unroll
    for (int i = 0; i < kSpBL; i++) {
        const uint32_t tok = min(tok0 + (uint32_t)i * 32u + (tid >> 3), p.tokens - 1u);
        off_b[i] = (tok - tok0) * p.ld_x * 2u + (tid & 7u) * 16u;
    }
#pragma unroll
    for (int i = 0; i < kSpAL; i++) {
        const uint32_t row = min(row0 + (uint32_t)i * 64u + (tid >> 2), p.rows - 1u);
        off_a[i] = (row - row0) * p.cols + (tid & 3u) * 16u;
    }
    const uint32_t i_row = min(row0 + (tid % kSpTR), p.rows - 1u);     // idx: 8 B per row and step
    const unsigned char *base_i = (const unsigned char *)p.idx + (size_t)row0 * (p.cols >> 3);
    const uint32_t off_i = (i_row - row0) * (p.cols >> 3);
    // The loads of step s + 1 are in flight while step s is multiplied; they then move from registers into
    // the other LDS buffer.  (A second register set, two steps ahead, measured no faster: the loop is bound
    // by load and LDS throughput, not by latency.)  Steps past the end re-read the last one with the A
    // values zeroed, so the loop body has no branch.
    struct Stage {
        su32x4 ra[kSpAL], rb[kSpBL];
        su32x2 ri;
    };
    Stage st[1];
    const uint32_t steps = p.cols / kSpKS;
    auto fetch = [&](Stage &r, uint32_t step) {
        const uint32_t k0 = min(step, steps - 1u) * kSpKS;
        // compressed A: cols/2 values per row = cols bytes per row; a step covers 32 values = 64 bytes
#pragma unroll
        for (int i = 0; i < kSpAL; i++)
            r.ra[i] = *(const su32x4 *)(base_a + k0 + off_a[i]);
#pragma unroll
        for (int i = 0; i < kSpBL; i++)
            r.rb[i] = *(const su32x4 *)(base_b + (size_t)k0 * 2u + off_b[i]);
        r.ri = *(const su32x2 *)(base_i + (k0 >> 3) + off_i);      // every thread loads (rows repeat if the tile has fewer than 256)
    };
    auto stash = [&](const Stage &r, int buf, uint32_t step) {
        const uint32_t live = step < steps ? 0xFFFFFFFFu : 0u;
#pragma unroll
        for (int i = 0; i < kSpAL; i++) {
            unsigned char *da = &As[buf][((uint32_t)i * 64u + (tid >> 2)) * kSpAPitch + (tid & 3u) * 16u];
            *(su32x2 *)(da) = su32x2{r.ra[i].x & live, r.ra[i].y & live};      // rows are 8-byte aligned only (pitch 72)
            *(su32x2 *)(da + 8) = su32x2{r.ra[i].z & live, r.ra[i].w & live};
        }
#pragma unroll
        for (int i = 0; i < kSpBL; i++)
            *(su32x4 *)&Bs[buf][((uint32_t)i * 32u + (tid >> 3)) * kSpBPitch + (tid & 7u) * 16u] = r.rb[i];
        *(su32x2 *)&Is[buf][(tid % kSpTR) * kSpIPitch] = r.ri;             // several writers of a row write the same bytes
    };

    f32x4 acc[kSpRT][kSpCT];
#pragma unroll
    for (int i = 0; i < kSpRT; i++)
#pragma unroll
        for (int j = 0; j < kSpCT; j++)
            acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    const uint32_t m = lane & 15u, a = lane >> 4;
    // the lane's two runs of compressed A inside a step: groups g0, g0+1 (8 bytes) and g0+4, g0+5
    const uint32_t g0 = 8u * (a & 1u) + 2u * (a >> 1);
    const uint32_t a_off = g0 * 4u;                 // bytes: 2 values x 2 bytes per group
    const uint32_t i_off = g0 >> 1;                 // index byte of groups g0, g0+1; groups g0+4, g0+5 are 2 further

    auto multiply = [&](int cur) {
        // B fragments of the wavefront's four token tiles
        bf16x16 bfrag[kSpCT];
#pragma unroll
        for (int ct = 0; ct < kSpCT; ct++) {
            const unsigned char *src = &Bs[cur][(wc * (kSpCT * 16u) + ct * 16u + m) * kSpBPitch + a * 32u];
            union { su32x4 u[2]; bf16x16 v; } cv;
            cv.u[0] = *(const su32x4 *)src;
            cv.u[1] = *(const su32x4 *)(src + 16);
            bfrag[ct] = cv.v;
        }
#pragma unroll
        for (int rt = 0; rt < kSpRT; rt++) {
            const uint32_t r = wr * (kSpRT * 16u) + rt * 16u + m;
            const unsigned char *src = &As[cur][r * kSpAPitch + a_off];
            union { su32x2 u[2]; bf16x8 v; } av;
            av.u[0] = *(const su32x2 *)src;
            av.u[1] = *(const su32x2 *)(src + 16);
            const unsigned char *is = &Is[cur][r * kSpIPitch + i_off];
            const int sel = (int)((uint32_t)is[0] | ((uint32_t)is[2] << 8));
#pragma unroll
            for (int ct = 0; ct < kSpCT; ct++)
                acc[rt][ct] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(av.v, bfrag[ct], acc[rt][ct], sel, 0, 0);
        }
    };

    fetch(st[0], 0);
    stash(st[0], 0, 0);
    __syncthreads();
    // The scheduler fences keep the order "issue loads, multiply, then wait for the loads and move them to
    // LDS": left alone, the compiler hoists the LDS writes (and with them the wait on the loads) above the
    // multiplications.
    for (uint32_t s = 0; s < steps; s += 2) {
        fetch(st[0], s + 1);
        __builtin_amdgcn_sched_barrier(0);
        multiply(0);
        __builtin_amdgcn_sched_barrier(0);
        stash(st[0], 1, s + 1);
        __syncthreads();
        fetch(st[0], s + 2);
        __builtin_amdgcn_sched_barrier(0);
        multiply(1);                  // step s + 1, all zeros in A if it lies past the end
        __builtin_amdgcn_sched_barrier(0);
        stash(st[0], 0, s + 2);
        __syncthreads();
    }

    // ---- store: lane holds rows 4a..4a+3 of token column m of each tile: 4 consecutive y entries ----
#pragma unroll
    for (int rt = 0; rt < kSpRT; rt++) {
#pragma unroll
        for (int ct = 0; ct < kSpCT; ct++) {
            const uint32_t tok = tok0 + wc * (kSpCT * 16u) + ct * 16u + m;
            const uint32_t r = row0 + wr * (kSpRT * 16u) + rt * 16u + a * 4u;
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
    if (rows > 0x7FFFFFFFll || tokens > 0x7FFFFFFFll || ld_y > 0x7FFFFFFFll || cols > (1ll << 22) || ld_x > (1ll << 22))
        return fail(TMASK_ERR_SHAPE, "rows, tokens, ld_y must stay below 2^31, cols and ld_x at or below 2^22");
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

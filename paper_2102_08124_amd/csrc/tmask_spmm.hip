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
// Tiling: a workgroup computes 256 rows x 128 tokens with eight wavefronts in two roles.  Wavefronts 0-3
// multiply (2 x 2, each 128 x 64 = 8 x 4 instruction tiles, 128 accumulator registers): they only read
// fragments from LDS and issue matrix instructions.  Wavefronts 4-7 feed them: per step of k = 64 they move
// the compressed A tile (256 x 32 values + 256 x 8 index bytes) and the x tile (128 tokens x 64) from global
// memory through registers into a ring of three LDS buffers, with three register sets, so a load is in flight
// for three steps before it is needed.  One barrier per step joins the two roles; each SIMD holds one wavefront
// of each role, so the feeders' waits and LDS writes overlap the multipliers' matrix instructions.  A workgroup
// is persistent: it takes every G-th tile and treats their steps as one stream, so nothing drains between
// tiles.  LDS rows are padded so that fragment reads are conflict-free.
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

constexpr int kSpThreads = 512;      // 4 multiplying + 4 feeding wavefronts
constexpr int kSpFeed = 256;         // threads that move tiles
constexpr int kSpRing = 3;           // LDS buffers
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
__global__ __launch_bounds__(kSpThreads, 1) void spmm24_kernel(const SpmmArgs p)
{
    __shared__ __attribute__((aligned(16))) unsigned char As[kSpRing][kSpTR * kSpAPitch];
    __shared__ __attribute__((aligned(16))) unsigned char Bs[kSpRing][kSpTT * kSpBPitch];
    __shared__ __attribute__((aligned(16))) unsigned char Is[kSpRing][kSpTR * kSpIPitch];

    // The grid is one workgroup per compute unit (or per tile if there are fewer); workgroup b works through
    // tiles b, b + G, b + 2G, ... as ONE stream of steps, so the loads of a tile's first steps are in flight
    // while the previous tile is still being multiplied and stored.
    // Tile numbers -> output position: workgroups are handed to the eight XCDs round-robin (b % 8 with G a
    // multiple of 8), so give each XCD a contiguous range of tile numbers, and number the tiles so that 64
    // consecutive ones form an 8 x 8 block of the output: the workgroups that run on one XCD at the same time
    // then share a few row panels of Wd and token panels of x in its L2 instead of streaming one each.
    const uint32_t n_tiles = p.tiles_r * p.tiles_t;
    const uint32_t G = gridDim.x, b = blockIdx.x;
    const uint32_t my_tiles = (n_tiles - b + G - 1u) / G;       // b < G <= n_tiles
    const uint32_t steps = p.cols / kSpKS;
    const uint32_t total = my_tiles * steps;                    // steps of this workgroup's stream
    auto locate = [&](uint32_t j, uint32_t &row0, uint32_t &tok0) {
        uint32_t id = b + j * G;
        const uint32_t per = n_tiles / 8u;
        if (id < per * 8u)
            id = (id & 7u) * per + (id >> 3);
        constexpr uint32_t kGroup = 8;
        const uint32_t in_group = kGroup * p.tiles_t;
        const uint32_t group = id / in_group, rem = id - group * in_group;
        const uint32_t first_r = group * kGroup;
        const uint32_t group_rows = min(p.tiles_r - first_r, kGroup);
        const uint32_t tt = rem / group_rows;
        row0 = (first_r + (rem - tt * group_rows)) * kSpTR;
        tok0 = tt * kSpTT;
    };
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool feeder = wave >= 4u;

    if (feeder) {
        // ---- global -> registers -> LDS (rows and tokens past the edge re-read the last valid one) ----
        // Consecutive lanes fetch consecutive 16-byte pieces of one row, so every load instruction covers whole
        // runs: 8 lanes = the 128 bytes a token contributes to a step, 4 lanes = the 64 bytes of a row of
        // compressed A.  (One lane per row with several pieces each touches four times as many cache lines per
        // instruction and measured twice as slow overall.)
        // Addresses are a wavefront-uniform base (scalar registers) plus a 32-bit lane offset.
        const uint32_t tid = threadIdx.x & (kSpFeed - 1);          // index among the feeding threads
        const unsigned char *base_a, *base_b, *base_i;
        uint32_t off_b[kSpBL], off_a[kSpAL], off_i;
        auto set_tile = [&](uint32_t j) {
            uint32_t row0, tok0;
            locate(j, row0, tok0);
            base_a = (const unsigned char *)p.vals + (size_t)row0 * p.cols;
            base_b = (const unsigned char *)p.x + (size_t)tok0 * p.ld_x * 2u;
            base_i = (const unsigned char *)p.idx + (size_t)row0 * (p.cols >> 3);
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
            off_i = (i_row - row0) * (p.cols >> 3);
        };
        struct Stage {
            su32x4 ra[kSpAL], rb[kSpBL];
            su32x2 ri;
        };
        Stage st[kSpRing];
        uint32_t fj = 0, fk = 0;          // tile ordinal and k-step of the next fetch
        set_tile(0);
        // fetch the next step of the stream; past its end the last step is read again (and never consumed)
        auto fetch = [&](Stage &r) {
            const uint32_t k0 = fk * kSpKS;
            // compressed A: cols/2 values per row = cols bytes per row; a step covers 32 values = 64 bytes
#pragma unroll
            for (int i = 0; i < kSpAL; i++)
                r.ra[i] = *(const su32x4 *)(base_a + k0 + off_a[i]);
#pragma unroll
            for (int i = 0; i < kSpBL; i++)
                r.rb[i] = *(const su32x4 *)(base_b + (size_t)k0 * 2u + off_b[i]);
            r.ri = *(const su32x2 *)(base_i + (k0 >> 3) + off_i);
            // advance (address arithmetic only: no memory operation inside the branch)
            if (fk + 1u < steps) {
                fk++;
            } else if (fj + 1u < my_tiles) {
                fk = 0;
                fj++;
                set_tile(fj);
            }
        };
        auto stash = [&](const Stage &r, int buf) {
#pragma unroll
            for (int i = 0; i < kSpAL; i++) {
                unsigned char *da = &As[buf][((uint32_t)i * 64u + (tid >> 2)) * kSpAPitch + (tid & 3u) * 16u];
                *(su32x2 *)(da) = su32x2{r.ra[i].x, r.ra[i].y};      // rows are 8-byte aligned only (pitch 72)
                *(su32x2 *)(da + 8) = su32x2{r.ra[i].z, r.ra[i].w};
            }
#pragma unroll
            for (int i = 0; i < kSpBL; i++)
                *(su32x4 *)&Bs[buf][((uint32_t)i * 32u + (tid >> 3)) * kSpBPitch + (tid & 7u) * 16u] = r.rb[i];
            // index bytes regrouped as (0, 2, 4, 6, 1, 3, 5, 7): the two bytes a lane needs (groups g0, g0+1 and
            // g0+4, g0+5) then sit side by side and come with one 16-bit read
            *(su32x2 *)&Is[buf][(tid % kSpTR) * kSpIPitch] =
                su32x2{__builtin_amdgcn_perm(r.ri.y, r.ri.x, 0x06040200u), __builtin_amdgcn_perm(r.ri.y, r.ri.x, 0x07050301u)};
        };
        // Stream step g is multiplied out of LDS buffer g % 3 while the feeders write step g + 2 into buffer
        // (g + 2) % 3 (last read at step g - 1, before the previous barrier) and issue the loads of step g + 5
        // into the register set they have just emptied.  Both roles run the same number of barriers; each has
        // its own loop, unrolled by three so that buffers and register sets are static, and its own registers.
        fetch(st[0]);
        fetch(st[1]);
        stash(st[0], 0);
        stash(st[1], 1);
        fetch(st[2]);
        fetch(st[0]);
        fetch(st[1]);
        __syncthreads();
        auto feed = [&](int pos) {                    // pos = g % 3, a compile-time constant at every call
            const int nxt = (pos + 2) % kSpRing;
            stash(st[nxt], nxt);                      // step g + 2
            __builtin_amdgcn_sched_barrier(0);
            fetch(st[nxt]);                           // step g + 5
            __syncthreads();
        };
        uint32_t g = 0;
        for (; g + 3 <= total; g += 3) {
            feed(0);
            feed(1);
            feed(2);
        }
        if (g < total)
            feed(0);
        if (g + 1 < total)
            feed(1);
    } else {
        const uint32_t wr = (wave >> 1) & 1u, wc = wave & 1u;     // position of this wavefront in the tile
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
        const uint32_t i_off = 2u * a;                  // the lane's two index bytes in the regrouped order

        // Fragments of x for a step are read one step ahead (the ring buffer of step g + 1 is complete when step
        // g starts), and so is the first A fragment: the matrix instructions of a step start without waiting
        // for LDS, and the remaining A fragments arrive while they run.
        auto read_b1 = [&](int buf, int ct, bf16x16 &bfrag) {
            const unsigned char *src = &Bs[buf][(wc * (kSpCT * 16u) + (uint32_t)ct * 16u + m) * kSpBPitch + a * 32u];
            union { su32x4 u[2]; bf16x16 v; } cv;
            cv.u[0] = *(const su32x4 *)src;
            cv.u[1] = *(const su32x4 *)(src + 16);
            bfrag = cv.v;
        };
        auto read_b = [&](int buf, bf16x16 (&bfrag)[kSpCT]) {
#pragma unroll
            for (int ct = 0; ct < kSpCT; ct++)
                read_b1(buf, ct, bfrag[ct]);
        };
        auto read_a = [&](int buf, int rt, bf16x8 &av, int &sel) {
            const uint32_t r = wr * (kSpRT * 16u) + (uint32_t)rt * 16u + m;
            const unsigned char *src = &As[buf][r * kSpAPitch + a_off];
            union { su32x2 u[2]; bf16x8 v; } cv;
            cv.u[0] = *(const su32x2 *)src;
            cv.u[1] = *(const su32x2 *)(src + 16);
            av = cv.v;
            sel = (int)*(const uint16_t *)&Is[buf][r * kSpIPitch + i_off];
        };
        bf16x16 bcur[kSpCT];
        bf16x8 a0;
        int sel0;
        // A fragments travel through a ring of three register sets, read two instruction rows ahead of their use,
        // and the reads of the next step's x fragments are spread over the rows: every matrix instruction finds
        // its operands in registers, and LDS latency hides behind the 4 x 16 cycles of a row of instructions.
        // (Left to itself the compiler reads every fragment into the registers of the one before, i.e. after the
        // instructions that use those have issued, and waits for it.)
        auto multiply = [&](int cur) {
            const int nxt = (cur + 1) % kSpRing;
            bf16x16 bnext[kSpCT];
            bf16x8 a0n;
            int sel0n;
            bf16x8 av[3];
            int sel[3];
            av[0] = a0;
            sel[0] = sel0;
            read_a(cur, 1, av[1], sel[1]);
            read_a(cur, 2, av[2], sel[2]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int rt = 0; rt < kSpRT; rt++) {
#pragma unroll
                for (int ct = 0; ct < kSpCT; ct++)
                    acc[rt][ct] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(av[rt % 3], bcur[ct], acc[rt][ct], sel[rt % 3], 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (rt + 3 < kSpRT)
                    read_a(cur, rt + 3, av[rt % 3], sel[rt % 3]);
                if (rt < kSpCT)
                    read_b1(nxt, rt, bnext[rt]);
                if (rt == kSpCT)
                    read_a(nxt, 0, a0n, sel0n);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int ct = 0; ct < kSpCT; ct++)
                bcur[ct] = bnext[ct];
            a0 = a0n;
            sel0 = sel0n;
        };
        // lane holds rows 4a..4a+3 of token column m of each instruction tile: 4 consecutive y entries
        auto store_tile = [&](uint32_t j) {
            uint32_t row0, tok0;
            locate(j, row0, tok0);
#pragma unroll
            for (int rt = 0; rt < kSpRT; rt++) {
#pragma unroll
                for (int ct = 0; ct < kSpCT; ct++) {
                    const uint32_t tok = tok0 + wc * (kSpCT * 16u) + ct * 16u + m;
                    const uint32_t r = row0 + wr * (kSpRT * 16u) + rt * 16u + a * 4u;
                    if (tok < p.tokens && r < p.rows) {       // rows is a multiple of 4: the four entries are in or out together
                        const f32x4 v = acc[rt][ct];
                        if constexpr (OUT_BF16) {
                            // fp32 -> bf16, round to nearest even, by the hardware's packed conversion
                            typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
                            typedef float f32x2 __attribute__((ext_vector_type(2)));
                            union { bf16x2 h; uint32_t u; } c0, c1;
                            c0.h = __builtin_convertvector(f32x2{v.x, v.y}, bf16x2);
                            c1.h = __builtin_convertvector(f32x2{v.z, v.w}, bf16x2);
                            const su32x2 o = {c0.u, c1.u};
                            *(su32x2 *)((unsigned char *)p.y + ((size_t)tok * p.ld_y + r) * 2u) = o;
                        } else {
                            *(f32x4 *)((unsigned char *)p.y + ((size_t)tok * p.ld_y + r) * 4u) = v;
                        }
                    }
                    acc[rt][ct] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
            }
        };
        uint32_t mj = 0, mk = 0;          // tile ordinal and k-step being multiplied
        auto mult = [&](int pos) {
            multiply(pos);
            __syncthreads();
            if (++mk == steps) {          // the tile is complete: write it while the feeders run ahead
                store_tile(mj);
                mk = 0;
                mj++;
            }
        };
        __syncthreads();
        read_b(0, bcur);
        read_a(0, 0, a0, sel0);
        uint32_t g = 0;
        for (; g + 3 <= total; g += 3) {
            mult(0);
            mult(1);
            mult(2);
        }
        if (g < total)
            mult(0);
        if (g + 1 < total)
            mult(1);
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
    // one workgroup per compute unit, a multiple of 8 (the XCD count) when there are that many tiles
    const int cus = cu_count();
    uint32_t grid = n_tiles < (uint64_t)cus ? (uint32_t)n_tiles : (uint32_t)cus;
    if (grid >= 8)
        grid &= ~7u;
    hipStream_t stream = (hipStream_t)hip_stream;
    {
        ProfileScope prof(stream, true);
        if (out_dt == TMASK_BF16)
            hipLaunchKernelGGL(spmm24_kernel<true>, dim3(grid), dim3(kSpThreads), 0, stream, p);
        else
            hipLaunchKernelGGL(spmm24_kernel<false>, dim3(grid), dim3(kSpThreads), 0, stream, p);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return hip_fail(e, "spmm kernel launch");
    return TMASK_OK;
}

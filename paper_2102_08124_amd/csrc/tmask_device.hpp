// Device-side building blocks shared by the tmask kernels (gfx950 only).
//
// Data layout ("strip" layout).  A lane owns a 16-byte-wide column strip of a block-row: C = 4 fp32
// or 8 bf16 consecutive columns, all M rows.  Consecutive lanes own consecutive strips, so every
// global load instruction of a wavefront reads one contiguous 1 KiB run of a matrix row, and mask
// rows are written as contiguous 256 B / 512 B runs.
//   M*sizeof(elem) == 16 : one lane = one block            (fp32 M=4, bf16 M=8)
//   M*sizeof(elem)  > 16 : G = M/C adjacent lanes = one block (fp32 M=8: 2, M=16: 4; bf16 M=16: 2);
//                          column-direction work is lane-local, row-direction work crosses the G
//                          lanes with DPP quad permutes (G lanes are an aligned part of a quad)
//   M*sizeof(elem)  < 16 : one lane = B = 2 adjacent blocks (bf16 M=4)
// Strips of a matrix are numbered block-row-major; a workgroup handles 256 consecutive strips.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tmask {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Store with the non-temporal hint, for data this kernel does not read again.  (Plain stores look up to 10 %
// faster when a benchmark rewrites one output buffer over and over, because part of it then stays in the
// memory-side cache; with fresh output buffers they are 5-20 % slower than these.)
template <typename T>
__device__ __forceinline__ void stream_store(T v, T *p)
{
    __builtin_nontemporal_store(v, p);
}

constexpr int kF32 = 0;
constexpr int kBF16 = 1;
constexpr int kMaskU8 = 0;
constexpr int kMaskBits = 1;
constexpr int kThreads = 256;        // workgroup size of the streaming kernels
constexpr int kMaxBatch = 256;       // matrices per launch (descriptor table travels as kernel argument, 14 KiB)

// One matrix as the kernels see it, 56 bytes.  The table of a launch is passed by value: the kernel-argument
// segment takes tens of KiB (launches with 64 KiB of arguments were checked on the device), workgroups read only the
// entries their binary search touches, with scalar loads, and nothing has to be uploaded or allocated per call.
struct MatDev {
    const void *w;
    void *mask;
    void *aux;           // score: per-block objective base for this matrix (float*), else unused
    uint32_t ld;         // elements
    uint32_t mask_ld;    // bytes
    uint32_t spr;        // strips per block-row = cols / C
    uint32_t n_strips;   // spr * rows / M
    uint32_t div_mul;    // s / spr == (uint64(s) * div_mul) >> div_shift for s < 2^31
    uint32_t div_shift;
    uint32_t tile0;      // first workgroup of this matrix inside the launch
    uint32_t pad;
};

// Which matrix does workgroup `tile` belong to?  A binary search over the table costs a chain of dependent scalar
// loads before a workgroup can issue its first vector load (eight for 144 matrices: several percent of a workgroup's
// life).  The host therefore adds a coarse index: the workgroups of a launch are cut into at most 256 buckets of
// 2^shift, and entry b packs the matrix of the bucket's first workgroup (low half) with that of the next bucket's
// first workgroup (high half).  One load narrows the search to that range, usually a single matrix.
constexpr int kCoarse = 256;

struct CoarseIndex {
    uint32_t shift;
    uint32_t e[kCoarse];
};

struct BatchArgs {
    MatDev m[kMaxBatch];
    CoarseIndex ci;
    uint32_t n_mats;
    uint32_t K;          // pruned per row/column = M - N
    uint32_t N;
    uint32_t partial0;   // index of this launch's first partial in the workspace
    void *partials;      // workspace
};

// What a workgroup of the score kernels leaves for the second-stage reduction.
struct ScorePartial {
    double retained, total;
    unsigned long long kept, rowv, colv, rowne, colne;
};

static_assert(sizeof(BatchArgs) <= 16384, "descriptor table is sized to stay a small kernel argument");

template <int DT, int M>
struct Geo {
    static constexpr int ES = (DT == kF32) ? 4 : 2;          // element bytes
    static constexpr int C = 16 / ES;                        // columns per strip
    static constexpr int G = (M > C) ? M / C : 1;            // lanes per block
    static constexpr int B = (M < C) ? C / M : 1;            // blocks per lane
    static constexpr int CL = C / B;                         // columns of one block inside a lane
};

// ---- cross-lane helpers -------------------------------------------------------------------------

// Value of lane (lane ^ X) within the quad, X in {1,2,3}: DPP quad_perm.
template <int X>
__device__ __forceinline__ uint32_t quad_xor(uint32_t v)
{
    constexpr int ctrl = (X == 1) ? 0xB1 : (X == 2) ? 0x4E : 0x1B;   // [1,0,3,2] [2,3,0,1] [3,2,1,0]
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, ctrl, 0xF, 0xF, false);
}

// v + the value of lane (lane ^ X) within the quad.  The source lane always exists and every lane is enabled, so
// "0 where the source is missing" never applies; written that way the move folds into the add (v_add_u32_dpp).
template <int X>
__device__ __forceinline__ uint32_t quad_xor_sum(uint32_t v)
{
    constexpr int ctrl = (X == 1) ? 0xB1 : (X == 2) ? 0x4E : 0x1B;
    return v + (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, ctrl, 0xF, 0xF, true);
}

// max / min of a and the value that lane (lane ^ X) of the quad holds in o, the move folded into the operation the same
// way (v_max_u32_dpp / v_min_u32_dpp: one instruction, and no wait states between a move and its use).
template <int X>
__device__ __forceinline__ uint32_t quad_xor_max(uint32_t a, uint32_t o)
{
    constexpr int ctrl = (X == 1) ? 0xB1 : (X == 2) ? 0x4E : 0x1B;
    const uint32_t y = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)o, ctrl, 0xF, 0xF, true);
    return a > y ? a : y;
}

template <int X>
__device__ __forceinline__ uint32_t quad_xor_min(uint32_t a, uint32_t o)
{
    constexpr int ctrl = (X == 1) ? 0xB1 : (X == 2) ? 0x4E : 0x1B;
    const uint32_t y = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)o, ctrl, 0xF, 0xF, true);
    return a < y ? a : y;
}

// A wavefront-wide boolean: bit l = the predicate in lane l.  Held in a scalar register pair, so
// logic on it is scalar-ALU work.
typedef unsigned long long lanemask_t;

__device__ __forceinline__ lanemask_t lm(bool pred) { return __builtin_amdgcn_ballot_w64(pred); }
__device__ __forceinline__ bool lm_test(lanemask_t m) { return __builtin_amdgcn_inverse_ballot_w64(m); }

__device__ __forceinline__ lanemask_t maj3(lanemask_t x, lanemask_t y, lanemask_t z)
{
    return (x & y) | (z & (x | y));
}

// r += 1 in the lanes whose bit is set in m: one add-with-carry-in, the carry being the lane mask.
__device__ __forceinline__ void lm_inc(uint32_t &r, lanemask_t m)
{
    lanemask_t carry_out;
    asm("v_addc_co_u32_e64 %0, %1, 0, %0, %2" : "+v"(r), "=s"(carry_out) : "s"(m));
}

// r = 2 r + (1 in the lanes whose bit is set in m): shifts a flag into a bit word, one add-with-carry-in.
__device__ __forceinline__ void lm_shift_in(uint32_t &r, lanemask_t m)
{
    lanemask_t carry_out;
    asm("v_addc_co_u32_e64 %0, %1, %0, %0, %2" : "+v"(r), "=s"(carry_out) : "s"(m));
}

// Wavefront sums by DPP, in a fixed order (deterministic): quad, then the four quads of a row of 16
// lanes by row rotation, then the four rows through scalar reads.  All 64 lanes must be active.
// The result is uniform.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_read(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xF, 0xF, false);
}

__device__ __forceinline__ float wave_sum(float v)
{
    v += __uint_as_float(dpp_read<0xB1>(__float_as_uint(v)));    // quad_perm [1,0,3,2]
    v += __uint_as_float(dpp_read<0x4E>(__float_as_uint(v)));    // quad_perm [2,3,0,1]
    v += __uint_as_float(dpp_read<0x124>(__float_as_uint(v)));   // row_ror:4
    v += __uint_as_float(dpp_read<0x128>(__float_as_uint(v)));   // row_ror:8
    const uint32_t u = __float_as_uint(v);
    return (__uint_as_float(__builtin_amdgcn_readlane(u, 0)) + __uint_as_float(__builtin_amdgcn_readlane(u, 16))) +
           (__uint_as_float(__builtin_amdgcn_readlane(u, 32)) + __uint_as_float(__builtin_amdgcn_readlane(u, 48)));
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v)
{
    v += dpp_read<0xB1>(v);
    v += dpp_read<0x4E>(v);
    v += dpp_read<0x124>(v);
    v += dpp_read<0x128>(v);
    return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
           __builtin_amdgcn_readlane(v, 48);
}

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        v += __shfl_xor(v, off, 64);
    return v;
}

__device__ __forceinline__ unsigned long long wave_sum(unsigned long long v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        v += __shfl_xor(v, off, 64);
    return v;
}

// Sum over the workgroup in a fixed tree order (deterministic); result valid in thread 0.
template <typename T>
__device__ __forceinline__ T block_sum(T v, T *lds /* kThreads/64 entries */)
{
    v = wave_sum(v);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0)
        lds[wave] = v;
    __syncthreads();
    T r = lds[0];
#pragma unroll
    for (int k = 1; k < kThreads / 64; k++)
        r += lds[k];
    __syncthreads();
    return r;
}

// Workgroup sum of per-thread fp32 values: fp32 inside a wavefront, fp64 across wavefronts.
__device__ __forceinline__ double block_sum_f32(float v, double *lds /* kThreads/64 entries */)
{
    const float w = wave_sum(v);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0)
        lds[wave] = (double)w;
    __syncthreads();
    double r = lds[0];
#pragma unroll
    for (int k = 1; k < kThreads / 64; k++)
        r += lds[k];
    return r;
}

// ---- tile addressing ----------------------------------------------------------------------------

// Which matrix of the batch does workgroup `tile` belong to (largest m with tile0[m] <= tile).
__device__ __forceinline__ int find_matrix(const BatchArgs &a, uint32_t tile)
{
    const uint32_t e = a.ci.e[tile >> a.ci.shift];
    int lo = (int)(e & 0xFFFFu), hi = (int)(e >> 16);
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (a.m[mid].tile0 <= tile)
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo;
}

struct StripPos {
    uint32_t br;   // block-row
    uint32_t sc;   // strip column inside the block-row
};

__device__ __forceinline__ StripPos strip_pos(const MatDev &md, uint32_t s)
{
    StripPos p;
    p.br = (uint32_t)(((uint64_t)s * md.div_mul) >> md.div_shift);
    p.sc = s - p.br * md.spr;
    return p;
}

// ---- strip load / store -------------------------------------------------------------------------

// Loads the lane's strip: a[i][c] = |W| as an fp32 bit pattern (bf16 widened by << 16), i.e. the
// magnitude ordering key, and raw[i] = the untouched 16 bytes of row i.
template <int DT, int M>
__device__ __forceinline__ void load_strip(const MatDev &md, StripPos p, uint32_t (&a)[M][Geo<DT, M>::C],
                                           u32x4 (&raw)[M])
{
    constexpr int C = Geo<DT, M>::C;
    const char *base = (const char *)md.w + ((size_t)p.br * M * md.ld + (size_t)p.sc * C) * Geo<DT, M>::ES;
    const size_t row_bytes = (size_t)md.ld * Geo<DT, M>::ES;
#pragma unroll
    for (int i = 0; i < M; i++)
        raw[i] = __builtin_nontemporal_load((const u32x4 *)(base + i * row_bytes));
#pragma unroll
    for (int i = 0; i < M; i++) {
        const uint32_t d[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};
        if constexpr (DT == kF32) {
#pragma unroll
            for (int c = 0; c < 4; c++)
                a[i][c] = d[c] & 0x7FFFFFFFu;
        } else {
#pragma unroll
            for (int c = 0; c < 4; c++) {
                a[i][2 * c] = (d[c] << 16) & 0x7FFF0000u;
                a[i][2 * c + 1] = d[c] & 0x7FFF0000u;
            }
        }
    }
}

// Spread the low 4 bits of b into 4 bytes (bit k -> byte k, value 0/1).
__device__ __forceinline__ uint32_t bits_to_bytes4(uint32_t b)
{
    return (b | (b << 7) | (b << 14) | (b << 21)) & 0x01010101u;
}

__device__ __forceinline__ uint32_t bytes4_to_bits(uint32_t v)
{
    // any non-zero byte counts as kept
    uint32_t nz = ((v & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | v;       // bit 7 of each byte = byte != 0
    nz = (nz >> 7) & 0x01010101u;
    return (nz | (nz >> 7) | (nz >> 14) | (nz >> 21)) & 0xFu;
}

// Writes the lane's C keep-bits of each of the M rows (bit c of rowbits[i] = column c kept).
template <int DT, int M, int FMT>
__device__ __forceinline__ void store_mask(const MatDev &md, StripPos p, const uint32_t (&rowbits)[M])
{
    constexpr int C = Geo<DT, M>::C;
    if constexpr (FMT == kMaskU8) {
        char *base = (char *)md.mask + (size_t)p.br * M * md.mask_ld + (size_t)p.sc * C;
#pragma unroll
        for (int i = 0; i < M; i++) {
            if constexpr (C == 4) {
                stream_store(bits_to_bytes4(rowbits[i]), (uint32_t *)(base + (size_t)i * md.mask_ld));
            } else {
                u32x2 v;
                v.x = bits_to_bytes4(rowbits[i] & 0xFu);
                v.y = bits_to_bytes4(rowbits[i] >> 4);
                stream_store(v, (u32x2 *)(base + (size_t)i * md.mask_ld));
            }
        }
    } else {
        // BITS: C bits per lane and row. fp32 (C=4): the even lane of a pair writes one byte built
        // from both lanes; bf16 (C=8): every lane writes its byte.
        char *base = (char *)md.mask + (size_t)p.br * M * md.mask_ld + (((size_t)p.sc * C) >> 3);
#pragma unroll
        for (int i = 0; i < M; i++) {
            if constexpr (C == 8) {
                base[(size_t)i * md.mask_ld] = (char)rowbits[i];
            } else {
                uint32_t other = quad_xor<1>(rowbits[i]);
                if ((threadIdx.x & 1) == 0)
                    base[(size_t)i * md.mask_ld] = (char)(rowbits[i] | (other << 4));
            }
        }
    }
}

// Reads the lane's C mask entries of each row into bit c of rowbits[i].
template <int DT, int M, int FMT>
__device__ __forceinline__ void load_mask(const MatDev &md, StripPos p, uint32_t (&rowbits)[M])
{
    constexpr int C = Geo<DT, M>::C;
    if constexpr (FMT == kMaskU8) {
        const char *base = (const char *)md.mask + (size_t)p.br * M * md.mask_ld + (size_t)p.sc * C;
#pragma unroll
        for (int i = 0; i < M; i++) {
            if constexpr (C == 4) {
                rowbits[i] = bytes4_to_bits(
                    __builtin_nontemporal_load((const uint32_t *)(base + (size_t)i * md.mask_ld)));
            } else {
                u32x2 v = __builtin_nontemporal_load((const u32x2 *)(base + (size_t)i * md.mask_ld));
                rowbits[i] = bytes4_to_bits(v.x) | (bytes4_to_bits(v.y) << 4);
            }
        }
    } else {
        const unsigned char *base =
            (const unsigned char *)md.mask + (size_t)p.br * M * md.mask_ld + (((size_t)p.sc * C) >> 3);
#pragma unroll
        for (int i = 0; i < M; i++) {
            uint32_t v = base[(size_t)i * md.mask_ld];
            if constexpr (C == 8)
                rowbits[i] = v;
            else
                rowbits[i] = (v >> ((p.sc & 1) * 4)) & 0xFu;
        }
    }
}

// Sum of the kept magnitudes of the lane's strip (fp32 within the strip).
template <int M, int C>
__device__ __forceinline__ float kept_sum(const uint32_t (&a)[M][C], const uint32_t (&rowbits)[M])
{
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < M; i++)
#pragma unroll
        for (int c = 0; c < C; c++)
            s += ((rowbits[i] >> c) & 1u) ? __uint_as_float(a[i][c]) : 0.f;
    return s;
}

}  // namespace tmask

/*
 * tmask -- N:M transposable sparsity masks on AMD MI355X (gfx950), C ABI.
 *
 * Implements the mask-computation path of "Accelerated Sparse Neural Training: A Provable and
 * Efficient Method to Find N:M Transposable Masks" (arXiv 2102.08124), Sec. 4:
 * a weight matrix is cut into M x M blocks (grid origin (0,0), stride M both ways) and a binary
 * mask S is computed per block so that both W and W^T obey the N:M pattern.
 *
 * Conventions
 *   N            entries KEPT per row and per column of a block (Eq. 3: row/column sums of S are N);
 *                K = M - N entries are pruned.  Supported: M in {4, 8, 16, 32}, 0 < N < M.
 *   S_ij = 1     W_ij is kept (Eq. 3).
 *   magnitude    |W_ij| is ordered by its bit pattern with the sign cleared, compared as an unsigned
 *                integer: -0 == +0, denormals are not flushed, +Inf > finite, NaN > Inf.
 *   tie-break    equal magnitudes are ordered by the row-major index i*M + j inside the block.
 *
 * Memory and execution
 *   Every `w`, `mask`, `vals*`, `idx*`, `objective`, `out`, `per_block_obj` and `workspace` pointer
 *   is DEVICE memory owned by the caller; descriptor arrays (`tmask_mat*`, `tmask_pack_desc*`, `tmask_fused_desc*`
 *   and the other `*_desc` types) are HOST memory read before the call returns.  Work is enqueued on `hip_stream` (a hipStream_t,
 *   NULL = default stream); the library never synchronises, allocates or frees device memory, and
 *   holds no state between calls (two documented exceptions: the one-shot events of tmask_profile_next, which are
 *   thread-local, and the static scratch array of tmask_approx_noalloc).  Outputs are valid once the stream has
 *   been synchronised.
 *   The workspace (at least tmask_workspace_bytes(), 256-byte aligned) is scratch for the duration
 *   of the enqueued work; calls that overlap on different streams need different workspaces.
 *
 * Layout requirements (checked; violations return TMASK_ERR_SHAPE / TMASK_ERR_ALIGN)
 *   rows and cols multiples of M (the paper's only requirement: Sec. 4 speaks of the M x M blocks of a weight
 *   matrix); ld >= cols (ld in elements); ld, mask_ld < 2^31; rows/M * ceil(cols/4) < 2^31; every pointer aligned
 *   to its element type.  U8 mask: mask_ld >= cols.  BITS mask: cols a multiple of 8, mask_ld >= cols/8 bytes.
 *   Packed outputs are dense (no leading dimension).
 * Fast and slow paths (same results, bit for bit where the result is unique)
 *   The streaming kernels read 16-byte strips: they need `w` 16-byte aligned with ld*sizeof(element) and
 *   cols*sizeof(element) multiples of 16 (ld, cols multiples of 4 for fp32, of 8 for bf16), a U8 mask pointer and
 *   mask_ld that are multiples of 4 (fp32) or 8 (bf16) bytes, packed value arrays 4-byte aligned (8-byte for the
 *   one-pass tmask_approx_pack kernels), dense outputs 16-byte aligned with a 16-byte pitch.  A call in which some
 *   matrix misses any of this, and every call with M = 32 (tmask_apply_pack at 16:32 with `vals` 16-byte aligned
 *   excepted), runs on element-wise kernels instead (one lane per column of a block): correct for every layout above, bound by the vector ALU or by LDS traffic instead of by
 *   memory.
 *
 * Errors
 *   All argument errors are detected on the host before anything is enqueued and leave the outputs
 *   untouched.  A mask that violates N:M is a *result* of tmask_score, never an error.
 *   tmask_last_error() returns a thread-local, human-readable description of the last failure.
 */
#ifndef TMASK_H
#define TMASK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { TMASK_F32 = 0, TMASK_BF16 = 1 } tmask_dtype;

/* TMASK_MASK_U8  : one byte per weight (0 or 1), row-major, row stride mask_ld bytes.
 * TMASK_MASK_BITS: one bit per weight, bit (c % 8) of byte [r*mask_ld + c/8], LSB first. */
typedef enum { TMASK_MASK_U8 = 0, TMASK_MASK_BITS = 1 } tmask_mask_fmt;

enum {
    TMASK_OK = 0,
    TMASK_ERR_NULL = -1,      /* a required pointer is NULL */
    TMASK_ERR_SHAPE = -2,     /* sizes <= 0, rows/cols not multiples of M, ld < cols, too many blocks */
    TMASK_ERR_NM = -3,        /* need M in {4,8,16,32} and 0 < N < M */
    TMASK_ERR_DTYPE = -4,     /* unknown dtype or mask format */
    TMASK_ERR_WORKSPACE = -5, /* workspace NULL, misaligned or smaller than tmask_workspace_bytes() */
    TMASK_ERR_HIP = -6,       /* a HIP call failed; text in tmask_last_error() */
    TMASK_ERR_ALIGN = -7      /* a pointer that is not aligned to its element type (see layout requirements) */
};

/* One 2-D weight matrix and where its mask goes. */
typedef struct {
    const void *w;     /* device, rows x cols elements of the call's dtype, row stride ld elements */
    int64_t rows, cols, ld;
    void *mask;        /* device; written by tmask_approx/tmask_exact, read by tmask_score */
    int64_t mask_ld;   /* bytes */
    double *objective; /* device, nullable: [0] <- retained L1 = sum_ij S_ij |W_ij| (Eq. 3's objective) */
} tmask_mat;

/*
 * Greedy 2-approximation (Sec. 4, Algorithm 1) on every block of every matrix, one batched launch
 * sequence.  Result per block: the set P of pruned entries produced by sweeping the block's entries
 * from light to heavy and taking an entry while its row or its column still has fewer than K
 * pruned entries; S = 1 - P.  P covers every row and column at least K times, so S keeps AT MOST N
 * per row and column (it is not repaired to exactly N).  Bit-deterministic: the same input gives
 * the same mask on every run, equal to a literal sort-and-sweep under the (magnitude, index) order.
 */
int tmask_approx(const tmask_mat *mats, int n_mats, tmask_dtype dt, int N, int M, tmask_mask_fmt mf,
                 void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * tmask_approx for callers that cannot allocate device memory and have no workspace to hand over: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus the workspace), same
 * kernels and bit-identical results as tmask_approx; the per-workgroup partial sums of the objectives go to a
 * 512 KiB array that lives inside the library's device code (one copy per GPU, kept until the process ends) instead
 * of a caller workspace.  The call allocates and frees nothing, on the host side of HIP or on the device.
 * Limit: at most 65536 workgroups of 256 strips over the whole batch when any objective is requested, i.e.
 * sum over matrices of ceil(rows/M * cols/C / 256) <= 65536 with C = 4 (fp32) or 8 (bf16) columns per strip
 * (268 M fp32 or 536 M bf16 weights at M = 4; proportionally more at M = 8, 16); beyond that TMASK_ERR_WORKSPACE is
 * returned before anything is enqueued.  Without objectives there is no limit.
 * All calls on one GPU share that array: calls that overlap in time on one GPU (different streams or threads) race
 * on the objectives (the masks are unaffected); calls enqueued on one stream are safe.
 */
int tmask_approx_noalloc(const tmask_mat *mats, int n_mats, tmask_dtype dt, int N, int M, tmask_mask_fmt mf,
                         void *hip_stream);

/*
 * Optimal mask of Eq. 3 per block (Sec. 4, the reduction to a min-cost flow, Fig. 3): exactly N kept
 * per row and column, maximum retained L1.  4 x 4 blocks are solved by evaluating all feasible
 * patterns in fp32 (90 at 2:4, the 24 permutations at 1:4 and 3:4); M >= 8 by successive shortest augmenting paths on the bipartite
 * row/column network with magnitudes truncated per block to 27 (M<=8), 26 (M=16) or 25 (M=32) significant
 * bits below the block maximum, which costs less than M*(M-N)*2^-26 (resp. 2^-25, 2^-24) of the block
 * maximum in retained L1 (below 1e-5 relative for M <= 16; at M = 32 below 6e-5 in the worst case and
 * about 1e-7 on real-valued data).  Among equally good
 * masks the choice is deterministic but unspecified.  Inputs must be finite for optimality; with
 * NaN/Inf present the mask is still valid (exactly N per row/column).
 */
int tmask_exact(const tmask_mat *mats, int n_mats, tmask_dtype dt, int N, int M, tmask_mask_fmt mf,
                void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Structured (non-transposable) N:M magnitude pruning, the baseline the paper compares with (Sec. 3,
 * constraint 2 of the mask-diversity list; Sec. 2): in every group of M consecutive elements of a row
 * the N heaviest are kept, order = (magnitude, position) as in tmask_approx, so W is N:M sparse along
 * its rows while W^T in general is not.  Same arguments, layout requirements, mask formats and
 * objective (sum S|W|) as tmask_approx; blocks play no role beyond rows % M == 0, cols % M == 0.
 */
int tmask_prune_1d(const tmask_mat *mats, int n_mats, tmask_dtype dt, int N, int M, tmask_mask_fmt mf,
                   void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Apply a mask and compress both operands the two training matmuls read (Sec. 1, Eq. 1, the
 * backward pass: forward uses W, backward uses W^T; Sec. 4: N non-zeros per M contiguous elements
 * in both).  The paper fixes no storage format; this one is the library's own:
 *   W (.) S is a select (pruned entries become +0, also when W_ij is NaN or Inf).
 *   vals  : rows x (cols*N/M) elements, row-major, dense.  Group g of row r (columns gM..gM+M-1)
 *           owns slots [g*N, g*N+N): the kept entries in ascending column order; if fewer than N
 *           are kept (possible for approximate masks) the lowest-numbered unused positions are added
 *           as +0 fillers and all N slots are ordered by position.
 *   idx   : per row, one ceil(log2 M)-bit position per slot, slot-major, LSB-first in little-endian
 *           bytes; row stride ceil(cols*N/M * log2(M) / 8) bytes.
 *   valsT, idxT: the same for W^T (cols x rows), i.e. groups are M consecutive rows of one column.
 * A group with more than N kept entries is a caller error (tmask_score reports it); the first N win.
 */
typedef struct {
    const void *w; int64_t rows, cols, ld;
    const void *mask; int64_t mask_ld;
    void *vals;  void *idx;
    void *valsT; void *idxT;
} tmask_pack_desc;

int tmask_apply_pack(const tmask_pack_desc *descs, int n, tmask_dtype dt, int N, int M, tmask_mask_fmt mf,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Algorithm 1 and the compression in one call (arXiv 2102.08124, Sec. 4: Algorithm 1; Sec. 1, Eq. 1: the
 * backward pass multiplies by W^T, so both W and W^T are compressed).  Outputs are exactly those of
 * tmask_approx followed by tmask_apply_pack with that mask: `vals`, `idx`, `valsT`, `idxT` in the
 * format above, `objective` (device, nullable) = sum S|W|, and the mask itself if `mask` is not
 * NULL.  For N:M = 2:4 and 4:8 (both types) this is a single pass over W in which the
 * mask never travels through memory (`mask` may be NULL for all matrices; give it for all or for
 * none, else TMASK_ERR_NULL).  For any other (type, N:M) the two steps run one after the other
 * and `mask` is required (TMASK_ERR_NULL without it).
 * A workspace is needed only if some `objective` is given.  The `w`, mask and packed-output layout
 * requirements are those of tmask_approx and tmask_apply_pack; for 2:4, `vals` and `valsT` must
 * be 8-byte aligned for the one-pass kernels; a call whose matrices or outputs miss that (or the alignment of the
 * strip kernels, see above) takes the two-step path (and then needs `mask`).
 */
typedef struct {
    const void *w; int64_t rows, cols, ld;
    void *mask; int64_t mask_ld;          /* output, nullable (see above) */
    void *vals;  void *idx;
    void *valsT; void *idxT;
    double *objective;                    /* output, nullable */
} tmask_fused_desc;

int tmask_approx_pack(const tmask_fused_desc *descs, int n, tmask_dtype dt, int N, int M, tmask_mask_fmt mf,
                      void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Score a mask (Eq. 3's objective and constraints).  out[m] (device) receives, for matrix m:
 * retained_l1 = sum S|W|, total_l1 = sum |W|, kept = sum S, row_violations / col_violations =
 * number of (block,row) / (block,column) pairs with more than N kept, row_not_n / col_not_n =
 * pairs whose kept count differs from N (zero for an exact-solver mask).
 * per_block_obj (device, nullable): retained L1 of every block as fp32, matrices concatenated in
 * call order, each block-row-major.  mats[m].objective is ignored.
 */
typedef struct {
    double retained_l1, total_l1;
    uint64_t kept, row_violations, col_violations, row_not_n, col_not_n;
} tmask_score_out;

int tmask_score(const tmask_mat *mats, int n_mats, tmask_dtype dt, int N, int M, tmask_mask_fmt mf,
                tmask_score_out *out, float *per_block_obj,
                void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Product with a compressed 2:4 operand on the structured-sparse matrix cores (arXiv 2102.08124,
 * Sec. 1 and Sec. 4: the forward pass multiplies by W, the backward pass by W^T (Eq. 1); with a
 * transposable mask both are 2:4 sparse along the reduction dimension):
 *
 *     y[t][r] = sum_c x[t][c] * Wd[r][c]      t < tokens, r < rows
 *
 * where Wd (rows x cols) is the matrix whose compressed form (vals, idx) was written by
 * tmask_apply_pack or tmask_approx_pack with N:M = 2:4 and bf16 weights.
 *   forward : (vals,  idx,  rows = W.rows, cols = W.cols), x = activations [tokens][W.cols]
 *   backward: (valsT, idxT, rows = W.cols, cols = W.rows), x = dLoss/dY   [tokens][W.rows]
 * x is bf16, row-major with leading dimension ld_x (elements); y is fp32 or bf16 (out_dt), row-major
 * with leading dimension ld_y.  Products are exact, sums are accumulated in fp32 in an unspecified
 * order.  All pointers are device memory.  No workspace.
 * Requirements (TMASK_ERR_SHAPE / TMASK_ERR_ALIGN): rows a multiple of 4, cols a multiple of 64,
 * ld_x >= cols and a multiple of 8, ld_y >= rows with ld_y*sizeof(y element) a multiple of 16;
 * vals, x, y 16-byte aligned, idx 8-byte aligned.
 */
int tmask_spmm24(const void *vals, const void *idx, int64_t rows, int64_t cols,
                 const void *x, int64_t ld_x, void *y, int64_t ld_y, int64_t tokens,
                 tmask_dtype out_dt, void *hip_stream);

/*
 * Number of entries whose kept/pruned state differs between two masks of the same shape: the
 * mask-flip count of a training loop that recomputes its transposable mask as the weights move
 * (Sec. 4.1, training from scratch: the mask is extracted again every few iterations from the dense
 * copy of the weights; flips[0] / (rows*cols) is the flip fraction between two extractions).
 * mask_a, mask_b: device, format mf (U8: any non-zero byte = kept), leading dimensions in bytes;
 * flips: device, 8-byte aligned, receives the count.  No workspace; the count is exact.
 */
typedef struct {
    const void *mask_a; int64_t ld_a;
    const void *mask_b; int64_t ld_b;
    int64_t rows, cols;
    uint64_t *flips;
} tmask_flip_desc;

int tmask_flip_count(const tmask_flip_desc *descs, int n, tmask_mask_fmt mf, void *hip_stream);

/*
 * Pattern violations (Sec. 5): the number of active (non-zero) weights that a mask removes -- what forcing an
 * N:M pattern on an unstructured-sparse model costs (the paper sets N:M per layer so that few such flips are
 * needed).  count[0] <- #{(i,j): W_ij is not +-0 (NaN counts as active) and S_ij = 0}.  Any mask is accepted.
 * w, mask, count: device; ld in elements, mask_ld in bytes; mask in format mf; count 8-byte aligned.
 * Requirements: any rows, cols > 0 (BITS masks need cols to be a multiple of 8); w aligned to its element type.
 * The streaming kernel runs when cols is a multiple of 16 bytes' worth of elements, w and its row pitch are 16-byte
 * aligned and a U8 mask and its pitch are aligned to 4 (fp32) or 8 (bf16) bytes; a call in which some matrix misses
 * that is counted element by element, with the same result.  No workspace; exact.
 */
typedef struct {
    const void *w; int64_t ld;
    const void *mask; int64_t mask_ld;
    int64_t rows, cols;
    uint64_t *count;
} tmask_violation_desc;

int tmask_pattern_violations(const tmask_violation_desc *descs, int n, tmask_dtype dt, tmask_mask_fmt mf,
                             void *hip_stream);

/*
 * Dense masked copy: out = W (.) S in W's own type, pruned entries as +0 -- the masked weights a
 * training step multiplies with where the sparse products are emulated by dense ones (Sec. 4.1; the
 * dense copy W stays untouched and the mask is taken from it again later).  out may be w itself
 * (in place).  With absorb_mean != 0 the bias fix of Sec. 5 is applied on the way: in every group of
 * M consecutive entries of a row, the arithmetic mean of the group's pruned weights is added to each
 * of its kept weights; groups with nothing pruned or nothing kept are only masked.  The mean and the
 * sums are fp32 (pruned weights in position order inside 16-byte pieces, pieces combined pairwise);
 * bf16 results are rounded to nearest even.  Any mask is accepted (transposable, 1-D, unstructured):
 * neither N nor the pattern is checked.  Without absorb_mean, M is ignored.
 * w, mask, out: device; ld, ld_out in elements, mask_ld in bytes; mask in format mf.
 * Requirements (checked): any rows, cols > 0 (cols a multiple of M with absorb_mean, M in
 * {2, 4, 8, 16, 32}; of 8 for BITS masks); w and out aligned to the element type.  The streaming
 * kernel runs when cols is a multiple of 16 bytes' worth of elements, w, out and their row pitches
 * are 16-byte aligned and a U8 mask and its pitch are aligned to 4 (fp32) or 8 (bf16) bytes; a call
 * in which some matrix misses that takes an element-wise kernel (same masked copy; with absorb_mean
 * the group's pruned weights are summed pairwise over the whole group).  No workspace.
 */
typedef struct {
    const void *w; int64_t ld;
    const void *mask; int64_t mask_ld;
    void *out; int64_t ld_out;
    int64_t rows, cols;
} tmask_dense_desc;

int tmask_apply_dense(const tmask_dense_desc *descs, int n, tmask_dtype dt, int M, int absorb_mean,
                      tmask_mask_fmt mf, void *hip_stream);

/*
 * Algorithm 1 and the dense masked copy in one call (Sec. 4, Algorithm 1; Sec. 4.1: the training loop keeps a
 * dense copy of the weights and masks it before the forward pass): out <- W (.) S with S the mask tmask_approx
 * computes, in W's type, pruned entries +0.  `mask` is an OUTPUT here and may be NULL for all matrices (then no
 * mask is written; give it for all or for none, else TMASK_ERR_NULL); `out` may be `w` itself.  One pass over W.
 * Shape requirements are those of tmask_approx for `w` and the mask; ld_out >= cols.  (An `out` that is not 16-byte
 * aligned with a 16-byte pitch sends the call to the element-wise kernels, like an unaligned `w`.)  No workspace, no
 * objective.
 */
typedef struct {
    const void *w; int64_t ld;
    void *mask; int64_t mask_ld;          /* output, nullable (see above) */
    void *out; int64_t ld_out;
    int64_t rows, cols;
} tmask_mask_dense_desc;                  /* same layout as tmask_dense_desc; the mask is written here */

int tmask_approx_dense(const tmask_mask_dense_desc *descs, int n, tmask_dtype dt, int N, int M, tmask_mask_fmt mf,
                       void *hip_stream);

/*
 * Structured N:M pruning along rows and the dense masked copy in one call, optionally with the bias fix of
 * Sec. 5 (Sec. 3, constraint 2: in every group of M consecutive elements of a row the N heaviest are kept;
 * Sec. 5: a model is forced into the N:M pattern this way, and the mean of each group's pruned weights is absorbed
 * into its kept ones).  out <- what tmask_prune_1d followed by tmask_apply_dense(absorb_mean) gives, in one pass
 * over W; `mask` is an OUTPUT and may be NULL for all matrices; `out` may be `w` itself.  Requirements as for
 * tmask_approx_dense.  No workspace, no objective.
 */
int tmask_prune_1d_dense(const tmask_mask_dense_desc *descs, int n, tmask_dtype dt, int N, int M, int absorb_mean,
                         tmask_mask_fmt mf, void *hip_stream);

/*
 * Mask diversity (Sec. 3, Eq. 2): the number of masks a structure constraint admits on a tensor of
 * T elements at sparsity level N/M, as the paper's four closed forms; *log10_md (HOST pointer)
 * receives log10 of it (the counts overflow doubles already for small tensors).  Pure host arithmetic.
 * Here, as in the paper's Sec. 3, the forms are symmetric in which N of M entries are zero or kept.
 */
typedef enum { TMASK_MD_UNSTRUCTURED = 0, TMASK_MD_STRUCTURED = 1, TMASK_MD_TRANSPOSABLE = 2,
               TMASK_MD_SEQUENTIAL = 3 } tmask_md_kind;

int tmask_mask_diversity(tmask_md_kind kind, int N, int M, int64_t T, double *log10_md);

/*
 * Probability that a block of M independent entries, each prunable with probability rho, is N:M
 * sparse in the sense of Sec. 5 (at least N of the M can be pruned): Eq. 4, the upper tail of a
 * binomial distribution.  *prob is a HOST pointer.  Pure host arithmetic.  (The number of
 * "pattern violations" that forcing an N:M mask onto an unstructured-sparse W costs is what
 * tmask_pattern_violations returns for W and that mask.)
 */
int tmask_nm_sparse_probability(int N, int M, double rho, double *prob);

/* Upper bound of the workspace any call above needs for these matrices (0 on invalid arguments). */
size_t tmask_workspace_bytes(const tmask_mat *mats, int n_mats, int N, int M);

/*
 * Profiling aid (not part of the paper's method).  The next tmask_approx / tmask_exact /
 * tmask_score / tmask_apply_pack call made on this thread records `start_event` (a hipEvent_t) on
 * the call's stream immediately before its main kernel and `stop_event` immediately after it, so
 * hipEventElapsedTime gives that kernel's duration (for calls split into several launches: the last
 * launch).  One-shot; pass NULLs to cancel.  The events are the caller's.
 */
int tmask_profile_next(void *start_event, void *stop_event);

/* Thread-local text of the last error returned on this thread ("" if none). */
const char *tmask_last_error(void);

/* Library version: major*10000 + minor*100 + patch. */
int tmask_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TMASK_H */

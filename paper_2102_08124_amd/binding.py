"""Thin ctypes binding over libtmask.so (include/tmask.h).

Argument marshalling only: every step of the path runs in the HIP kernels.  PyTorch provides the
device memory (tensors) and the stream; nothing here computes on tensors.  There is no CPU
fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtmask.so")

TMASK_F32, TMASK_BF16 = 0, 1
TMASK_MASK_U8, TMASK_MASK_BITS = 0, 1
TMASK_OK = 0
TMASK_ERR_NULL, TMASK_ERR_SHAPE, TMASK_ERR_NM, TMASK_ERR_DTYPE = -1, -2, -3, -4
TMASK_ERR_WORKSPACE, TMASK_ERR_HIP, TMASK_ERR_ALIGN = -5, -6, -7

EXPORTS = ("tmask_approx", "tmask_approx_noalloc", "tmask_exact", "tmask_prune_1d", "tmask_apply_pack", "tmask_apply_dense", "tmask_approx_dense", "tmask_prune_1d_dense", "tmask_approx_pack", "tmask_spmm24", "tmask_flip_count", "tmask_pattern_violations", "tmask_mask_diversity", "tmask_nm_sparse_probability", "tmask_score",
           "tmask_workspace_bytes", "tmask_profile_next", "tmask_last_error", "tmask_version")


class tmask_violation_desc(C.Structure):
    _fields_ = [("w", C.c_void_p), ("ld", C.c_int64), ("mask", C.c_void_p), ("mask_ld", C.c_int64),
                ("rows", C.c_int64), ("cols", C.c_int64), ("count", C.c_void_p)]


class TmaskError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("tmask error %d: %s" % (code, text))
        self.code = code


class tmask_mat(C.Structure):
    _fields_ = [("w", C.c_void_p), ("rows", C.c_int64), ("cols", C.c_int64), ("ld", C.c_int64),
                ("mask", C.c_void_p), ("mask_ld", C.c_int64), ("objective", C.c_void_p)]


class tmask_pack_desc(C.Structure):
    _fields_ = [("w", C.c_void_p), ("rows", C.c_int64), ("cols", C.c_int64), ("ld", C.c_int64),
                ("mask", C.c_void_p), ("mask_ld", C.c_int64),
                ("vals", C.c_void_p), ("idx", C.c_void_p), ("valsT", C.c_void_p), ("idxT", C.c_void_p)]


class tmask_fused_desc(C.Structure):
    _fields_ = [("w", C.c_void_p), ("rows", C.c_int64), ("cols", C.c_int64), ("ld", C.c_int64),
                ("mask", C.c_void_p), ("mask_ld", C.c_int64),
                ("vals", C.c_void_p), ("idx", C.c_void_p), ("valsT", C.c_void_p), ("idxT", C.c_void_p),
                ("objective", C.c_void_p)]


class tmask_flip_desc(C.Structure):
    _fields_ = [("mask_a", C.c_void_p), ("ld_a", C.c_int64), ("mask_b", C.c_void_p), ("ld_b", C.c_int64),
                ("rows", C.c_int64), ("cols", C.c_int64), ("flips", C.c_void_p)]


class tmask_dense_desc(C.Structure):
    _fields_ = [("w", C.c_void_p), ("ld", C.c_int64), ("mask", C.c_void_p), ("mask_ld", C.c_int64),
                ("out", C.c_void_p), ("ld_out", C.c_int64), ("rows", C.c_int64), ("cols", C.c_int64)]


tmask_mask_dense_desc = tmask_dense_desc


class tmask_score_out(C.Structure):
    _fields_ = [("retained_l1", C.c_double), ("total_l1", C.c_double), ("kept", C.c_uint64),
                ("row_violations", C.c_uint64), ("col_violations", C.c_uint64),
                ("row_not_n", C.c_uint64), ("col_not_n", C.c_uint64)]


SCORE_OUT_BYTES = C.sizeof(tmask_score_out)
_lib = None


def load_library():
    """Loads libtmask.so; raises if it has not been built (python -m paper_2102_08124_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libtmask.so is missing: build it with `python -m paper_2102_08124_amd.build` "
                           "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    vp, ci, sz = C.c_void_p, C.c_int, C.c_size_t
    for name in ("tmask_approx", "tmask_exact", "tmask_prune_1d"):
        f = getattr(L, name)
        f.restype = ci
        f.argtypes = [C.POINTER(tmask_mat), ci, ci, ci, ci, ci, vp, sz, vp]
    L.tmask_approx_noalloc.restype = ci
    L.tmask_approx_noalloc.argtypes = [C.POINTER(tmask_mat), ci, ci, ci, ci, ci, vp]
    L.tmask_apply_pack.restype = ci
    L.tmask_apply_pack.argtypes = [C.POINTER(tmask_pack_desc), ci, ci, ci, ci, ci, vp, sz, vp]
    L.tmask_approx_pack.restype = ci
    L.tmask_approx_pack.argtypes = [C.POINTER(tmask_fused_desc), ci, ci, ci, ci, ci, vp, sz, vp]
    L.tmask_spmm24.restype = ci
    L.tmask_spmm24.argtypes = [vp, vp, C.c_int64, C.c_int64, vp, C.c_int64, vp, C.c_int64, C.c_int64, ci, vp]
    L.tmask_flip_count.restype = ci
    L.tmask_flip_count.argtypes = [C.POINTER(tmask_flip_desc), ci, ci, vp]
    L.tmask_apply_dense.restype = ci
    L.tmask_apply_dense.argtypes = [C.POINTER(tmask_dense_desc), ci, ci, ci, ci, ci, vp]
    L.tmask_approx_dense.restype = ci
    L.tmask_approx_dense.argtypes = [C.POINTER(tmask_dense_desc), ci, ci, ci, ci, ci, vp]
    L.tmask_prune_1d_dense.restype = ci
    L.tmask_prune_1d_dense.argtypes = [C.POINTER(tmask_dense_desc), ci, ci, ci, ci, ci, ci, vp]
    L.tmask_pattern_violations.restype = ci
    L.tmask_pattern_violations.argtypes = [C.POINTER(tmask_violation_desc), ci, ci, ci, vp]
    L.tmask_mask_diversity.restype = ci
    L.tmask_mask_diversity.argtypes = [ci, ci, ci, C.c_int64, C.POINTER(C.c_double)]
    L.tmask_nm_sparse_probability.restype = ci
    L.tmask_nm_sparse_probability.argtypes = [ci, ci, C.c_double, C.POINTER(C.c_double)]
    L.tmask_score.restype = ci
    L.tmask_score.argtypes = [C.POINTER(tmask_mat), ci, ci, ci, ci, ci, vp, vp, vp, sz, vp]
    L.tmask_workspace_bytes.restype = sz
    L.tmask_workspace_bytes.argtypes = [C.POINTER(tmask_mat), ci, ci, ci]
    L.tmask_profile_next.restype = ci
    L.tmask_profile_next.argtypes = [vp, vp]
    L.tmask_last_error.restype = C.c_char_p
    L.tmask_last_error.argtypes = []
    L.tmask_version.restype = ci
    L.tmask_version.argtypes = []
    _lib = L
    return L


def _check(rc: int):
    if rc != TMASK_OK:
        raise TmaskError(rc, load_library().tmask_last_error().decode())


def dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return TMASK_F32
    if t.dtype == torch.bfloat16:
        return TMASK_BF16
    raise TypeError("weights must be float32 or bfloat16, got %s" % t.dtype)


def _mat2d(t: torch.Tensor, what: str):
    if t.dim() != 2 or not t.is_cuda or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError("%s must be a 2-D CUDA tensor with unit column stride" % what)
    return t.data_ptr(), int(t.shape[0]), int(t.shape[1]), int(t.stride(0))


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def mask_shape(rows: int, cols: int, mask_fmt: int):
    return (rows, cols) if mask_fmt == TMASK_MASK_U8 else (rows, (cols + 7) // 8)


def alloc_masks(ws: Sequence[torch.Tensor], mask_fmt: int = TMASK_MASK_U8):
    return [torch.empty(mask_shape(w.shape[0], w.shape[1], mask_fmt), dtype=torch.uint8, device=w.device)
            for w in ws]


def _mats(ws, masks, objective) -> "C.Array":
    n = len(ws)
    if len(masks) != n:
        raise ValueError("one mask per matrix expected")
    if objective is not None and (objective.dtype != torch.float64 or objective.numel() < n
                                  or not objective.is_cuda or not objective.is_contiguous()):
        raise ValueError("objective must be a contiguous CUDA float64 tensor with one entry per matrix")
    arr = (tmask_mat * n)()
    for k, (w, m) in enumerate(zip(ws, masks)):
        p, r, c, ld = _mat2d(w, "w")
        if m.dtype != torch.uint8:
            raise TypeError("mask must be uint8")
        mp, _, _, mld = _mat2d(m, "mask")
        arr[k] = tmask_mat(p, r, c, ld, mp, mld, objective.data_ptr() + 8 * k if objective is not None else None)
    return arr


class MatBatch:
    """Host descriptor array for a batch of matrices, marshalled once and reusable across calls
    (keeps the tensors alive).  Pass it in place of `ws` (with masks=None) to tmask_approx /
    tmask_exact / tmask_score to skip per-call marshalling in tight loops."""

    def __init__(self, ws, masks, objective=None):
        self.ws, self.masks, self.objective = list(ws), list(masks), objective
        self.arr = _mats(self.ws, self.masks, objective)
        self.n = len(self.ws)
        self.dt = dtype_code(self.ws[0])
        if any(dtype_code(w) != self.dt for w in self.ws):
            raise TypeError("all matrices of one call share a dtype")


class PackBatch:
    """Host descriptor array for tmask_apply_pack, marshalled once (keeps the tensors alive)."""

    def __init__(self, ws, masks, packed, N: int, M: int):
        self.ws, self.masks, self.packed = list(ws), list(masks), list(packed)
        self.n = len(self.ws)
        self.dt = dtype_code(self.ws[0])
        self.arr = (tmask_pack_desc * self.n)()
        for k, (w, m, pk) in enumerate(zip(self.ws, self.masks, self.packed)):
            p, r, c, ld = _mat2d(w, "w")
            mp, _, _, mld = _mat2d(m, "mask")
            vs, is_, vts, its = packed_shapes(r, c, N, M)
            vals, idx, valsT, idxT = pk
            for t, shp, dty in ((vals, vs, w.dtype), (idx, is_, torch.uint8), (valsT, vts, w.dtype),
                                (idxT, its, torch.uint8)):
                if tuple(t.shape) != shp or t.dtype != dty or not t.is_contiguous() or not t.is_cuda:
                    raise ValueError("packed output has the wrong shape/dtype: %s vs %s" % (tuple(t.shape), shp))
            self.arr[k] = tmask_pack_desc(p, r, c, ld, mp, mld, vals.data_ptr(), idx.data_ptr(), valsT.data_ptr(),
                                          idxT.data_ptr())


class FusedBatch:
    """Host descriptor array for tmask_approx_pack, marshalled once (keeps the tensors alive).
    masks: list of mask tensors, or None (2:4 and 4:8 only: no mask is written).
    objective: float64 device tensor with one entry per matrix, or None."""

    def __init__(self, ws, masks, packed, N: int, M: int, objective: Optional[torch.Tensor] = None):
        self.ws, self.packed = list(ws), list(packed)
        self.masks = None if masks is None else list(masks)
        self.objective = objective
        self.n = len(self.ws)
        self.dt = dtype_code(self.ws[0])
        if objective is not None and (objective.dtype != torch.float64 or objective.numel() < self.n
                                      or not objective.is_cuda or not objective.is_contiguous()):
            raise ValueError("objective must be a contiguous float64 device tensor with one entry per matrix")
        self.arr = (tmask_fused_desc * self.n)()
        for k, (w, pk) in enumerate(zip(self.ws, self.packed)):
            p, r, c, ld = _mat2d(w, "w")
            mp, mld = None, 0
            if self.masks is not None:
                mp, _, _, mld = _mat2d(self.masks[k], "mask")
            vs, is_, vts, its = packed_shapes(r, c, N, M)
            vals, idx, valsT, idxT = pk
            for t, shp, dty in ((vals, vs, w.dtype), (idx, is_, torch.uint8), (valsT, vts, w.dtype),
                                (idxT, its, torch.uint8)):
                if tuple(t.shape) != shp or t.dtype != dty or not t.is_contiguous() or not t.is_cuda:
                    raise ValueError("packed output has the wrong shape/dtype: %s vs %s" % (tuple(t.shape), shp))
            op = None if objective is None else objective.data_ptr() + 8 * k
            self.arr[k] = tmask_fused_desc(p, r, c, ld, mp, mld, vals.data_ptr(), idx.data_ptr(), valsT.data_ptr(),
                                           idxT.data_ptr(), op)


def tmask_workspace_bytes(ws: Sequence[torch.Tensor], N: int, M: int) -> int:
    arr = (tmask_mat * len(ws))()
    for k, w in enumerate(ws):
        arr[k] = tmask_mat(None, int(w.shape[0]), int(w.shape[1]), int(w.stride(0)), None, 0, None)
    return int(load_library().tmask_workspace_bytes(arr, len(ws), N, M))


def alloc_workspace(ws: Sequence[torch.Tensor], N: int, M: int) -> torch.Tensor:
    return torch.empty(max(tmask_workspace_bytes(ws, N, M), 256), dtype=torch.uint8, device=ws[0].device)


def _ws_args(workspace):
    if workspace is None:
        return None, 0
    return C.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()


def _run_mask(fn, ws, masks, N, M, objective, mask_fmt, workspace, stream):
    b = ws if isinstance(ws, MatBatch) else MatBatch(ws, masks, objective)
    wp, wb = _ws_args(workspace)
    _check(fn(b.arr, b.n, b.dt, N, M, mask_fmt, wp, wb, _stream_ptr(stream)))


def tmask_approx(ws, masks, N: int, M: int, objective: Optional[torch.Tensor] = None,
                 mask_fmt: int = TMASK_MASK_U8, workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    """Algorithm 1 on every M x M block of every matrix; masks (and objective[k]) are written in place."""
    _run_mask(load_library().tmask_approx, ws, masks, N, M, objective, mask_fmt, workspace, stream)


def tmask_approx_noalloc(ws, masks, N: int, M: int, objective: Optional[torch.Tensor] = None,
                         mask_fmt: int = TMASK_MASK_U8, stream=None) -> None:
    """tmask_approx without a workspace: the partial sums live in the library's own static device array."""
    b = ws if isinstance(ws, MatBatch) else MatBatch(ws, masks, objective)
    _check(load_library().tmask_approx_noalloc(b.arr, b.n, b.dt, N, M, mask_fmt, _stream_ptr(stream)))


def tmask_exact(ws, masks, N: int, M: int, objective: Optional[torch.Tensor] = None,
                mask_fmt: int = TMASK_MASK_U8, workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    """Optimum of Eq. 3 on every block; masks (and objective[k]) are written in place."""
    _run_mask(load_library().tmask_exact, ws, masks, N, M, objective, mask_fmt, workspace, stream)


def tmask_prune_1d(ws, masks, N: int, M: int, objective: Optional[torch.Tensor] = None,
                   mask_fmt: int = TMASK_MASK_U8, workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    """Structured N:M magnitude pruning along rows (non-transposable baseline); same arguments as tmask_approx."""
    _run_mask(load_library().tmask_prune_1d, ws, masks, N, M, objective, mask_fmt, workspace, stream)


def tmask_score(ws, masks, N: int, M: int, out: torch.Tensor, per_block_obj: Optional[torch.Tensor] = None,
                mask_fmt: int = TMASK_MASK_U8, workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    """out: CUDA uint8 tensor of len(ws) * SCORE_OUT_BYTES bytes (array of tmask_score_out)."""
    b = ws if isinstance(ws, MatBatch) else MatBatch(ws, masks, None)
    if out.numel() * out.element_size() < b.n * SCORE_OUT_BYTES or not out.is_cuda or not out.is_contiguous():
        raise ValueError("out is too small")
    if per_block_obj is not None and (per_block_obj.dtype != torch.float32 or not per_block_obj.is_contiguous()):
        raise ValueError("per_block_obj must be contiguous float32")
    wp, wb = _ws_args(workspace)
    _check(load_library().tmask_score(b.arr, b.n, b.dt, N, M, mask_fmt, C.c_void_p(out.data_ptr()),
                                      C.c_void_p(per_block_obj.data_ptr()) if per_block_obj is not None else None,
                                      wp, wb, _stream_ptr(stream)))


def read_scores(out: torch.Tensor, n: int):
    """Copies the device array of tmask_score_out back and returns a list of dicts."""
    raw = out.cpu().numpy().tobytes()
    res = []
    for k in range(n):
        s = tmask_score_out.from_buffer_copy(raw, k * SCORE_OUT_BYTES)
        res.append({f: getattr(s, f) for f, _ in tmask_score_out._fields_})
    return res


def index_bits(M: int) -> int:
    return (M - 1).bit_length()


def packed_shapes(rows: int, cols: int, N: int, M: int):
    ib = index_bits(M)
    sw, st = cols // M * N, rows // M * N
    return (rows, sw), (rows, (sw * ib + 7) // 8), (cols, st), (cols, (st * ib + 7) // 8)


def alloc_packed(w: torch.Tensor, N: int, M: int):
    vs, is_, vts, its = packed_shapes(w.shape[0], w.shape[1], N, M)
    return (torch.empty(vs, dtype=w.dtype, device=w.device), torch.empty(is_, dtype=torch.uint8, device=w.device),
            torch.empty(vts, dtype=w.dtype, device=w.device), torch.empty(its, dtype=torch.uint8, device=w.device))


def tmask_apply_pack(ws, masks, packed, N: int, M: int, mask_fmt: int = TMASK_MASK_U8,
                     workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    """packed[k] = (vals, idx, valsT, idxT) tensors for matrix k (see alloc_packed), written in place."""
    b = ws if isinstance(ws, PackBatch) else PackBatch(ws, masks, packed, N, M)
    wp, wb = _ws_args(workspace)
    _check(load_library().tmask_apply_pack(b.arr, b.n, b.dt, N, M, mask_fmt, wp, wb, _stream_ptr(stream)))


def tmask_approx_pack(ws, masks, packed, N: int, M: int, objective: Optional[torch.Tensor] = None,
                      mask_fmt: int = TMASK_MASK_U8, workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    """Algorithm 1 and the compression of W and W^T in one call; masks may be None for 2:4 and for 4:8."""
    b = ws if isinstance(ws, FusedBatch) else FusedBatch(ws, masks, packed, N, M, objective)
    wp, wb = _ws_args(workspace)
    _check(load_library().tmask_approx_pack(b.arr, b.n, b.dt, N, M, mask_fmt, wp, wb, _stream_ptr(stream)))


def tmask_spmm24(vals: torch.Tensor, idx: torch.Tensor, rows: int, cols: int, x: torch.Tensor, y: torch.Tensor,
                 stream=None) -> None:
    """y[t][r] = sum_c x[t][c] * Wd[r][c] with Wd (rows x cols) given by its compressed 2:4 form (vals, idx).
    x: tokens x cols bfloat16 (row stride = leading dimension), y: tokens x rows float32 or bfloat16."""
    if x.dtype != torch.bfloat16 or vals.dtype != torch.bfloat16 or idx.dtype != torch.uint8:
        raise TypeError("vals and x must be bfloat16, idx uint8")
    if x.dim() != 2 or y.dim() != 2 or x.stride(1) != 1 or y.stride(1) != 1 or not (x.is_cuda and y.is_cuda):
        raise ValueError("x and y must be 2-D device tensors with unit column stride")
    if x.shape[1] != cols or tuple(y.shape) != (x.shape[0], rows):
        raise ValueError("shapes: x is tokens x cols, y is tokens x rows")
    if tuple(vals.shape) != (rows, cols // 2) or tuple(idx.shape) != (rows, cols // 8) or not vals.is_contiguous() \
            or not idx.is_contiguous():
        raise ValueError("vals must be rows x cols/2 and idx rows x cols/8, contiguous")
    _check(load_library().tmask_spmm24(vals.data_ptr(), idx.data_ptr(), rows, cols, x.data_ptr(), x.stride(0),
                                       y.data_ptr(), y.stride(0), x.shape[0], dtype_code(y), _stream_ptr(stream)))


MD_KINDS = {"unstructured": 0, "structured": 1, "transposable": 2, "sequential": 3}


def tmask_flip_count(masks_a, masks_b, cols, flips: torch.Tensor, mask_fmt: int = TMASK_MASK_U8, stream=None) -> None:
    """flips[k] (uint64 held in an int64 device tensor) = entries of masks_a[k] and masks_b[k] that differ in
    kept/pruned state.  cols[k] = logical columns of matrix k (the row length in entries)."""
    n = len(masks_a)
    if flips.dtype != torch.int64 or flips.numel() < n or not flips.is_cuda or not flips.is_contiguous():
        raise ValueError("flips must be a contiguous int64 device tensor with one entry per matrix")
    arr = (tmask_flip_desc * n)()
    for k, (a, b) in enumerate(zip(masks_a, masks_b)):
        pa, ra, _, lda = _mat2d(a, "mask_a")
        pb, rb, _, ldb = _mat2d(b, "mask_b")
        if ra != rb:
            raise ValueError("masks must have the same shape")
        arr[k] = tmask_flip_desc(pa, lda, pb, ldb, ra, int(cols[k]), flips.data_ptr() + 8 * k)
    _check(load_library().tmask_flip_count(arr, n, mask_fmt, _stream_ptr(stream)))


def tmask_pattern_violations(ws, masks, counts: torch.Tensor, mask_fmt: int = TMASK_MASK_U8, stream=None) -> None:
    """counts[k] (int64 device tensor) = number of non-zero entries of ws[k] that masks[k] removes (Sec. 5)."""
    n = len(ws)
    if counts.dtype != torch.int64 or counts.numel() < n or not counts.is_contiguous():
        raise ValueError("counts must be a contiguous int64 tensor with one entry per matrix")
    arr = (tmask_violation_desc * n)()
    dt = dtype_code(ws[0])
    for k, (w, m) in enumerate(zip(ws, masks)):
        if dtype_code(w) != dt:
            raise ValueError("all matrices of a call share one dtype")
        pw, rows, cols, ld = _mat2d(w, "w")
        pm, mr, _, mld = _mat2d(m, "mask")
        if mr != rows:
            raise ValueError("w and mask must describe the same matrix")
        arr[k] = tmask_violation_desc(pw, ld, pm, mld, rows, cols, counts.data_ptr() + 8 * k)
    _check(load_library().tmask_pattern_violations(arr, n, dt, mask_fmt, _stream_ptr(stream)))


def tmask_apply_dense(ws, masks, outs, M: int = 0, absorb_mean: bool = False, mask_fmt: int = TMASK_MASK_U8,
                      stream=None) -> None:
    """outs[k] = ws[k] masked by masks[k], in the weights' dtype (outs[k] may be ws[k]); with absorb_mean the mean
    of the pruned weights of every group of M along a row is added to the group's kept weights."""
    n = len(ws)
    arr = (tmask_dense_desc * n)()
    dt = dtype_code(ws[0])
    for k, (w, m, o) in enumerate(zip(ws, masks, outs)):
        if dtype_code(w) != dt or o.dtype != w.dtype:
            raise ValueError("all matrices and outputs of a call share one dtype")
        pw, rows, cols, ld = _mat2d(w, "w")
        pm, mr, _, mld = _mat2d(m, "mask")
        po, orows, ocols, old = _mat2d(o, "out")
        if (orows, ocols) != (rows, cols) or mr != rows:
            raise ValueError("w, mask and out must describe the same matrix")
        arr[k] = tmask_dense_desc(pw, ld, pm, mld, po, old, rows, cols)
    _check(load_library().tmask_apply_dense(arr, n, dt, M, 1 if absorb_mean else 0, mask_fmt, _stream_ptr(stream)))


def _dense_descs(ws, masks, outs):
    """Descriptors for the calls that write a masked copy and, optionally, the mask they computed."""
    n = len(ws)
    arr = (tmask_dense_desc * n)()
    dt = dtype_code(ws[0])
    for k, (w, o) in enumerate(zip(ws, outs)):
        if dtype_code(w) != dt or o.dtype != w.dtype:
            raise ValueError("all matrices and outputs of a call share one dtype")
        pw, rows, cols, ld = _mat2d(w, "w")
        po, orows, ocols, old = _mat2d(o, "out")
        if (orows, ocols) != (rows, cols):
            raise ValueError("w and out must describe the same matrix")
        pm, mld = None, 0
        if masks is not None:
            pm, mr, _, mld = _mat2d(masks[k], "mask")
            if mr != rows:
                raise ValueError("w and mask must describe the same matrix")
        arr[k] = tmask_dense_desc(pw, ld, pm, mld, po, old, rows, cols)
    return arr, n, dt


class DenseBatch:
    """Host descriptor array for tmask_approx_dense / tmask_prune_1d_dense, marshalled once (keeps the tensors alive).
    masks: list of mask tensors to be written, or None."""

    def __init__(self, ws, masks, outs):
        self.ws, self.outs = list(ws), list(outs)
        self.masks = None if masks is None else list(masks)
        self.arr, self.n, self.dt = _dense_descs(self.ws, self.masks, self.outs)


def tmask_approx_dense(ws, masks, outs, N: int, M: int, mask_fmt: int = TMASK_MASK_U8, stream=None) -> None:
    """Algorithm 1 and the masked copy in one pass: outs[k] = ws[k] with the entries Algorithm 1 prunes set to +0
    (outs[k] may be ws[k]); masks[k] receives the mask, or masks is None and no mask is written.  `ws` may be a
    DenseBatch (then masks and outs are ignored)."""
    arr, n, dt = (ws.arr, ws.n, ws.dt) if isinstance(ws, DenseBatch) else _dense_descs(ws, masks, outs)
    _check(load_library().tmask_approx_dense(arr, n, dt, N, M, mask_fmt, _stream_ptr(stream)))


def tmask_prune_1d_dense(ws, masks, outs, N: int, M: int, absorb_mean: bool = False,
                         mask_fmt: int = TMASK_MASK_U8, stream=None) -> None:
    """N:M pruning along rows and the masked copy in one pass (outs[k] may be ws[k]); with absorb_mean the mean of
    every row group's pruned weights is added to its kept ones.  masks[k] receives the mask, or masks is None.  `ws` may
    be a DenseBatch."""
    arr, n, dt = (ws.arr, ws.n, ws.dt) if isinstance(ws, DenseBatch) else _dense_descs(ws, masks, outs)
    _check(load_library().tmask_prune_1d_dense(arr, n, dt, N, M, 1 if absorb_mean else 0, mask_fmt, _stream_ptr(stream)))


def tmask_mask_diversity(kind: str, N: int, M: int, T: int) -> float:
    """log10 of the number of masks the constraint admits on T elements at sparsity N/M (host arithmetic)."""
    out = C.c_double(0.0)
    _check(load_library().tmask_mask_diversity(MD_KINDS[kind], N, M, T, C.byref(out)))
    return out.value


def tmask_nm_sparse_probability(N: int, M: int, rho: float) -> float:
    """P(at least N of M i.i.d. entries are prunable), each with probability rho (host arithmetic)."""
    out = C.c_double(0.0)
    _check(load_library().tmask_nm_sparse_probability(N, M, float(rho), C.byref(out)))
    return out.value


def tmask_profile_next(start_event: Optional[int], stop_event: Optional[int]) -> None:
    """hipEvent_t handles (as integers) recorded around the main kernel of the next call; None cancels."""
    _check(load_library().tmask_profile_next(C.c_void_p(start_event), C.c_void_p(stop_event)))


def tmask_version() -> int:
    return int(load_library().tmask_version())

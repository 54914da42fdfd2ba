"""ctypes front-end to the C oracle (test infrastructure; see tmask_oracle.c for what it computes).

Arrays: fp32 matrices are ``np.float32``; bfloat16 matrices are raw bit patterns in ``np.uint16``.
Masks are ``np.uint8`` (1 = kept).  N = kept per row/column of an M x M block (Eq. 3).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

F32, BF16 = 0, 1
_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tmask_oracle.c")
_SO = os.path.join(_HERE, "libtmask_oracle.so")
_lib = None


def lib_path() -> str:
    return _SO


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (no hand vectorisation, no tuning)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        tmp = _SO + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-fPIC", "-shared", "-pthread",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _SO)
    return _SO


def _load():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_SO)
        i64, vp, ci = C.c_int64, C.c_void_p, C.c_int
        for name in ("oracle_approx", "oracle_exact"):
            f = getattr(L, name)
            f.restype = ci
            f.argtypes = [vp, ci, i64, i64, i64, ci, ci, vp, i64, vp, vp, ci]
        L.oracle_score.restype = ci
        L.oracle_score.argtypes = [vp, ci, i64, i64, i64, ci, ci, vp, i64, vp, vp, vp]
        L.oracle_apply_pack.restype = ci
        L.oracle_apply_pack.argtypes = [vp, ci, i64, i64, i64, ci, ci, vp, i64, vp, vp, vp, vp]
        L.oracle_unpack.restype = ci
        L.oracle_unpack.argtypes = [vp, vp, ci, i64, i64, ci, ci, vp]
        L.oracle_prune_1d.restype = ci
        L.oracle_prune_1d.argtypes = [vp, ci, i64, i64, i64, ci, ci, vp, i64, vp]
        L.oracle_network_sizes.restype = None
        L.oracle_network_sizes.argtypes = [ci, ci, vp]
        _lib = L
    return _lib


def _dtype_of(w: np.ndarray) -> int:
    if w.dtype == np.float32:
        return F32
    if w.dtype == np.uint16:
        return BF16
    raise TypeError("oracle takes float32 matrices or uint16 bfloat16 bit patterns, got %s" % w.dtype)


def _prep(w: np.ndarray):
    if w.ndim != 2:
        raise ValueError("2-D matrix expected")
    w = np.ascontiguousarray(w)
    return w, _dtype_of(w)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError("%s failed with status %d" % (what, rc))


def _run_mask(fn_name, w, N, M, threads, want_blocks):
    w, dt = _prep(w)
    rows, cols = w.shape
    mask = np.zeros((rows, cols), dtype=np.uint8)
    obj = np.zeros(1, dtype=np.float64)
    pb = np.zeros((rows // M) * (cols // M) if (want_blocks and M > 0) else 0, dtype=np.float64)
    rc = getattr(_load(), fn_name)(_ptr(w), dt, rows, cols, cols, N, M, _ptr(mask), cols, _ptr(obj),
                                   _ptr(pb) if want_blocks else None, threads)
    _check(rc, fn_name)
    if want_blocks:
        return mask, float(obj[0]), pb.reshape(rows // M, cols // M)
    return mask, float(obj[0])


def approx(w: np.ndarray, N: int, M: int, threads: int = 1, per_block: bool = False):
    """Algorithm 1 on every M x M block -> (mask, retained L1[, per-block retained L1])."""
    return _run_mask("oracle_approx", w, N, M, threads, per_block)


def exact(w: np.ndarray, N: int, M: int, threads: int = 1, per_block: bool = False):
    """Optimum of Eq. 3 on every block via the Fig. 3 min-cost flow -> (mask, retained L1[, per-block])."""
    return _run_mask("oracle_exact", w, N, M, threads, per_block)


@dataclass
class Score:
    retained_l1: float
    total_l1: float
    kept: int
    row_violations: int   # (block,row) pairs with more than N kept
    col_violations: int
    row_not_n: int        # (block,row) pairs with kept != N
    col_not_n: int
    per_block: np.ndarray


def score(w: np.ndarray, mask: np.ndarray, N: int, M: int) -> Score:
    w, dt = _prep(w)
    rows, cols = w.shape
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    if mask.shape != w.shape:
        raise ValueError("mask shape mismatch")
    out = np.zeros(2, dtype=np.float64)
    cnt = np.zeros(5, dtype=np.uint64)
    pb = np.zeros((rows // M) * (cols // M), dtype=np.float64)
    _check(_load().oracle_score(_ptr(w), dt, rows, cols, cols, N, M, _ptr(mask), cols, _ptr(out), _ptr(cnt),
                                _ptr(pb)), "oracle_score")
    return Score(float(out[0]), float(out[1]), int(cnt[0]), int(cnt[1]), int(cnt[2]), int(cnt[3]), int(cnt[4]),
                 pb.reshape(rows // M, cols // M))


def index_bits(M: int) -> int:
    b = 0
    while (1 << b) < M:
        b += 1
    return b


def packed_shapes(rows: int, cols: int, N: int, M: int):
    """(vals shape, idx shape, valsT shape, idxT shape); idx arrays are bytes."""
    ib = index_bits(M)
    sw, st = cols // M * N, rows // M * N
    return (rows, sw), (rows, (sw * ib + 7) // 8), (cols, st), (cols, (st * ib + 7) // 8)


def apply_pack(w: np.ndarray, mask: np.ndarray, N: int, M: int):
    """W (.) S, then compress W and W^T -> (vals, idx, valsT, idxT)."""
    w, dt = _prep(w)
    rows, cols = w.shape
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    vs, is_, vts, its = packed_shapes(rows, cols, N, M)
    vals, valsT = np.zeros(vs, dtype=w.dtype), np.zeros(vts, dtype=w.dtype)
    idx, idxT = np.zeros(is_, dtype=np.uint8), np.zeros(its, dtype=np.uint8)
    _check(_load().oracle_apply_pack(_ptr(w), dt, rows, cols, cols, N, M, _ptr(mask), cols, _ptr(vals), _ptr(idx),
                                     _ptr(valsT), _ptr(idxT)), "oracle_apply_pack")
    return vals, idx, valsT, idxT


def unpack(vals: np.ndarray, idx: np.ndarray, R: int, Ccols: int, N: int, M: int) -> np.ndarray:
    """Dense R x Ccols matrix from a packed operand (zeros where nothing is stored)."""
    vals = np.ascontiguousarray(vals)
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    dt = _dtype_of(vals)
    dense = np.zeros((R, Ccols), dtype=vals.dtype)
    _check(_load().oracle_unpack(_ptr(vals), _ptr(idx), dt, R, Ccols, N, M, _ptr(dense)), "oracle_unpack")
    return dense


def prune_1d(w: np.ndarray, N: int, M: int):
    """Structured N:M magnitude pruning along rows (groups of M consecutive elements keep their N heaviest)
    -> (mask, retained L1).  The non-transposable baseline of Sec. 3."""
    w, dt = _prep(w)
    rows, cols = w.shape
    mask = np.zeros((rows, cols), dtype=np.uint8)
    obj = np.zeros(1, dtype=np.float64)
    _check(_load().oracle_prune_1d(_ptr(w), dt, rows, cols, w.strides[0] // w.itemsize, N, M, _ptr(mask), cols,
                                   _ptr(obj)), "oracle_prune_1d")
    return mask, float(obj[0])


def apply_dense(w: np.ndarray, mask: np.ndarray, M: int = 0, absorb_mean: bool = False) -> np.ndarray:
    """The masked weights W (.) S as a dense fp64 matrix (Sec. 4: what a training step multiplies with when the
    hardware product is emulated).  With absorb_mean, the bias fix of Sec. 5: in every group of M consecutive
    entries of a row, the arithmetic mean of the pruned weights is added to each kept weight (groups with
    nothing pruned, or nothing kept, change nothing beyond the masking)."""
    w = np.asarray(w, dtype=np.float64)
    keep = np.asarray(mask) != 0
    out = np.where(keep, w, 0.0)
    if absorb_mean:
        rows, cols = w.shape
        for r in range(rows):
            for g in range(0, cols, M):
                k = keep[r, g:g + M]
                n_pruned = int((~k).sum())
                if n_pruned == 0 or n_pruned == M:
                    continue
                mean = float(w[r, g:g + M][~k].sum()) / n_pruned
                out[r, g:g + M][k] += mean
    return out


def flip_count(mask_a: np.ndarray, mask_b: np.ndarray) -> int:
    """Number of entries whose kept (non-zero) / pruned (zero) state differs between two masks."""
    return int(((np.asarray(mask_a) != 0) != (np.asarray(mask_b) != 0)).sum())


def pattern_violations(w: np.ndarray, mask: np.ndarray) -> int:
    """Pattern violations of Sec. 5: active (non-zero) weights that the mask removes -- what forcing an N:M pattern on
    an unstructured-sparse model costs.  -0 counts as zero, NaN as non-zero; bf16 weights come as uint16 bit patterns."""
    w = np.asarray(w)
    if w.dtype == np.uint16:
        nonzero = (w & np.uint16(0x7FFF)) != 0
    else:
        nonzero = (w.view(np.uint32) & np.uint32(0x7FFFFFFF)) != 0 if w.dtype == np.float32 else (w != 0) | np.isnan(w)
    return int((nonzero & (np.asarray(mask) == 0)).sum())


def mask_diversity_log10(kind: str, N: int, M: int, T: int) -> float:
    """log10 of the mask diversity of Sec. 3 (Eq. 2) in exact integer arithmetic.
    kind: 'unstructured' | 'structured' | 'transposable' | 'sequential'; T = tensor size, sparsity N/M."""
    import math
    if kind == "unstructured":
        md = math.comb(T, N * T // M)
    elif kind == "structured":
        md = math.comb(M, N) ** (T // M)
    elif kind == "transposable":
        per_block = 1
        for q in range(N):
            per_block *= math.factorial(M - q)            # M! (M-1)! ... (M-N+1)!
        md = per_block ** (T // (M * M))
    elif kind == "sequential":
        md = (M - N + 1) ** (T // M)
    else:
        raise ValueError(kind)
    return math.log10(md)


def nm_sparse_probability(N: int, M: int, rho) -> float:
    """Sec. 5, Eq. 4 in exact rational arithmetic: sum_{i >= N} C(M, i) rho^i (1 - rho)^(M - i)."""
    import math
    from fractions import Fraction
    r = Fraction(rho)
    return float(sum(math.comb(M, i) * r ** i * (1 - r) ** (M - i) for i in range(N, M + 1)))


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float64, exactly."""
    return (np.ascontiguousarray(bits).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def spmm(vals: np.ndarray, idx: np.ndarray, rows: int, cols: int, N: int, M: int, x: np.ndarray) -> np.ndarray:
    """y[t][r] = sum_c x[t][c] * Wd[r][c] in float64, Wd = the rows x cols matrix stored as (vals, idx):
    the forward product of Sec. 1 / Eq. 1's backward product, depending on which packed operand is passed.
    The definition written out: expand the operand (oracle_unpack), then one float64 matrix product.
    x: tokens x cols, float32 or bfloat16 bit patterns."""
    wd = unpack(vals, idx, rows, cols, N, M)
    wd = bf16_to_f64(wd) if wd.dtype == np.uint16 else wd.astype(np.float64)
    xf = bf16_to_f64(x) if x.dtype == np.uint16 else np.asarray(x).astype(np.float64)
    return xf @ wd.T


def network_sizes(N: int, M: int):
    """(nodes, edges, demand) of the Fig. 3 network the exact solver builds."""
    out = np.zeros(3, dtype=np.int64)
    _load().oracle_network_sizes(N, M, _ptr(out))
    return int(out[0]), int(out[1]), int(out[2])

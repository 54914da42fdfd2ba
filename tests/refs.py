"""Independent yardsticks the oracle is pinned to (numpy / scipy / networkx; tests only).

Nothing here is derived from the oracle's code: each function is either a plain definition
(enumeration of Eq. 3's feasible set), a library routine solving the same mathematical problem
(LP, assignment, network simplex), or a characterisation proved separately (per-node K lightest).
"""
from __future__ import annotations

import itertools

import numpy as np


def magnitude_keys(w: np.ndarray) -> np.ndarray:
    """Ordering key of |w|: bit pattern with the sign cleared (fp32 or raw bf16 bits)."""
    if w.dtype == np.float32:
        return w.view(np.uint32) & np.uint32(0x7FFFFFFF)
    if w.dtype == np.uint16:
        return (w & np.uint16(0x7FFF)).astype(np.uint32)
    raise TypeError(w.dtype)


def magnitudes(w: np.ndarray) -> np.ndarray:
    if w.dtype == np.float32:
        return np.abs(w.astype(np.float64))
    if w.dtype == np.uint16:
        return np.abs(((w.astype(np.uint32) & np.uint32(0x7FFF)) << np.uint32(16)).view(np.float32).astype(np.float64))
    raise TypeError(w.dtype)


def to_blocks(a: np.ndarray, M: int) -> np.ndarray:
    """rows x cols -> (block_rows, block_cols, M, M)."""
    r, c = a.shape
    return a.reshape(r // M, M, c // M, M).transpose(0, 2, 1, 3)


def from_blocks(b: np.ndarray) -> np.ndarray:
    br, bc, M, _ = b.shape
    return b.transpose(0, 2, 1, 3).reshape(br * M, bc * M)


def k_lightest_rule(w: np.ndarray, N: int, M: int) -> np.ndarray:
    """Mask that keeps (i,j) iff it is NOT among the K lightest of its block-row and NOT among the
    K lightest of its block-column, under the (magnitude, row-major index) order.

    For Algorithm 1 with the strict degree test this is provably the same set: the n-th lightest
    edge at a node (n <= K) meets fewer than K pruned edges there and is taken; an edge outside
    the K lightest at both ends finds both ends saturated.
    """
    K = M - N
    keys = to_blocks(magnitude_keys(w), M).astype(np.int64)
    pos = np.arange(M * M, dtype=np.int64).reshape(M, M)
    full = keys * (M * M) + pos                       # strict total order inside a block
    row_rank = np.argsort(np.argsort(full, axis=3), axis=3)
    col_rank = np.argsort(np.argsort(full, axis=2), axis=2)
    keep = (row_rank >= K) & (col_rank >= K)
    return from_blocks(keep.astype(np.uint8))


def valid_patterns(N: int, M: int) -> np.ndarray:
    """All 0/1 M x M matrices with every row sum and column sum equal to N (Eq. 3's feasible set)."""
    rows = [np.array([1 if j in c else 0 for j in range(M)], dtype=np.int8)
            for c in itertools.combinations(range(M), N)]
    out = []

    def rec(i, col_sum, chosen):
        if i == M:
            if np.all(col_sum == N):
                out.append(np.stack(chosen))
            return
        remaining = M - i - 1
        for r in rows:
            cs = col_sum + r
            if np.any(cs > N) or np.any(cs + remaining < N):
                continue
            rec(i + 1, cs, chosen + [r])

    rec(0, np.zeros(M, dtype=np.int64), [])
    return np.stack(out).astype(np.uint8)


def brute_force_best(w: np.ndarray, N: int, M: int, patterns: np.ndarray | None = None) -> np.ndarray:
    """Per-block maximum of sum S|W| over all valid patterns -> (block_rows, block_cols) fp64."""
    if patterns is None:
        patterns = valid_patterns(N, M)
    a = to_blocks(magnitudes(w), M)
    br, bc = a.shape[:2]
    scores = a.reshape(br * bc, M * M) @ patterns.reshape(len(patterns), M * M).T.astype(np.float64)
    return scores.max(axis=1).reshape(br, bc)


def lp_best(block_abs: np.ndarray, N: int) -> float:
    """max sum S|W| s.t. row/col sums = N, 0 <= S <= 1, solved as an LP by HiGHS.  The constraint
    matrix (bipartite incidence) is totally unimodular, so the LP optimum equals Eq. 3's."""
    from scipy.optimize import linprog
    M = block_abs.shape[0]
    A = np.zeros((2 * M, M * M))
    for i in range(M):
        A[i, i * M:(i + 1) * M] = 1.0
        A[M + i, i::M] = 1.0
    res = linprog(-block_abs.reshape(-1), A_eq=A, b_eq=np.full(2 * M, float(N)), bounds=(0.0, 1.0), method="highs")
    assert res.status == 0
    return float(-res.fun)


def per_block_sums(a: np.ndarray, M: int) -> np.ndarray:
    return to_blocks(a, M).sum(axis=(2, 3))


def unpack_indices(idx_row: np.ndarray, n_slots: int, bits: int) -> np.ndarray:
    """Slots of `bits` bits, LSB-first, from a little-endian byte row."""
    allbits = np.unpackbits(idx_row, bitorder="little")
    need = n_slots * bits
    return (allbits[:need].reshape(n_slots, bits).astype(np.int64) << np.arange(bits)).sum(axis=1)

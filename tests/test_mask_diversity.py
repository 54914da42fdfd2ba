"""Mask diversity (Sec. 3, Eq. 2): the oracle's exact integer arithmetic against the values the paper prints in
Table 1, and the library's host routine against the oracle.  CPU only."""
import numpy as np
import math
import os

import pytest

import oracle
from paper_2102_08124_amd import binding as tm

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "mask_diversity_table1.txt")


def _table():
    rows = []
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            kind, n, m, v = line.split()
            rows.append((kind, int(n), int(m), float(v)))
    return rows


def test_oracle_reproduces_table_1():
    rows = _table()
    assert len(rows) == 12
    for kind, N, M, printed in rows:
        got = oracle.mask_diversity_log10(kind, N, M, 64)
        assert abs(got - math.log10(printed)) < math.log10(1.1), (kind, N, M, 10 ** got, printed)


def test_oracle_closed_forms_by_counting():
    # brute-force counts on tiny tensors pin the forms that are true counts
    import itertools
    # structured 1:2 on T = 4: each pair has C(2,1) = 2 masks -> 4
    assert round(10 ** oracle.mask_diversity_log10("structured", 1, 2, 4)) == 4
    # unstructured: choose T/2 of T
    assert round(10 ** oracle.mask_diversity_log10("unstructured", 1, 2, 6)) == math.comb(6, 3)
    # sequential 2:4 on one group: runs of 2 zeros can start at 3 places
    assert round(10 ** oracle.mask_diversity_log10("sequential", 2, 4, 4)) == 3
    # transposable 1:2 on one 2x2 block: permutation matrices -> 2 (the paper's form M!...(M-N+1)! = 2! here)
    count = sum(1 for bits in itertools.product((0, 1), repeat=4)
                if bits[0] + bits[1] == 1 and bits[2] + bits[3] == 1 and bits[0] + bits[2] == 1 and bits[1] + bits[3] == 1)
    assert count == 2 == round(10 ** oracle.mask_diversity_log10("transposable", 1, 2, 4))


@pytest.mark.parametrize("kind", ["unstructured", "structured", "transposable", "sequential"])
@pytest.mark.parametrize("N,M", [(1, 2), (2, 4), (4, 8), (8, 16), (1, 4), (3, 8)])
def test_library_matches_oracle(kind, N, M):
    for T in (M * M, 64 * M * M):       # exact big-integer arithmetic on the oracle side: keep T moderate
        got = tm.tmask_mask_diversity(kind, N, M, T)
        want = oracle.mask_diversity_log10(kind, N, M, T)
        assert got == pytest.approx(want, rel=1e-10, abs=1e-9)


def test_library_argument_errors():
    with pytest.raises(tm.TmaskError) as e:
        tm.tmask_mask_diversity("structured", 4, 4, 64)
    assert e.value.code == tm.TMASK_ERR_NM
    with pytest.raises(tm.TmaskError) as e:
        tm.tmask_mask_diversity("transposable", 2, 4, 24)
    assert e.value.code == tm.TMASK_ERR_SHAPE


# ---- Sec. 5, Eq. 4: probability that a block is N:M sparse ----

def test_probability_closed_forms_pin_the_oracle():
    from fractions import Fraction
    assert oracle.nm_sparse_probability(1, 2, Fraction(1, 2)) == 0.75                 # 1 - P(no prunable entry)
    assert oracle.nm_sparse_probability(0, 8, Fraction(1, 3)) == 1.0
    assert oracle.nm_sparse_probability(8, 8, Fraction(1, 2)) == 0.5 ** 8
    assert oracle.nm_sparse_probability(4, 8, Fraction(1, 2)) == pytest.approx(163 / 256, rel=1e-15)   # (1 + C(8,4)/2^8)/2
    # complement symmetry: P(at least N | rho) + P(at least M-N+1 | 1-rho) = 1
    for N, M, rho in ((2, 4, Fraction(3, 10)), (5, 8, Fraction(43, 50)), (9, 16, Fraction(1, 7))):
        assert oracle.nm_sparse_probability(N, M, rho) + oracle.nm_sparse_probability(M - N + 1, M, 1 - rho) == \
            pytest.approx(1.0, abs=1e-15)
    # brute force over all 2^M outcomes on a small block
    import itertools
    rho = 0.86
    want = sum(rho ** sum(o) * (1 - rho) ** (6 - sum(o)) for o in itertools.product((0, 1), repeat=6) if sum(o) >= 4)
    assert oracle.nm_sparse_probability(4, 6, Fraction(43, 50)) == pytest.approx(want, rel=1e-13)


@pytest.mark.parametrize("N,M", [(1, 2), (2, 4), (4, 8), (6, 8), (8, 16), (0, 4), (4, 4), (100, 256)])
def test_probability_library_matches_oracle(N, M):
    from fractions import Fraction
    for rho in (Fraction(0), Fraction(1, 2), Fraction(43, 50), Fraction(1), Fraction(1, 100)):
        assert tm.tmask_nm_sparse_probability(N, M, float(rho)) == pytest.approx(oracle.nm_sparse_probability(N, M, rho),
                                                                                 rel=1e-10, abs=1e-300)
    with pytest.raises(tm.TmaskError):
        tm.tmask_nm_sparse_probability(5, 4, 0.5)


# ---------------------------------------------------------------- pattern violations (Sec. 5) -------------------

def test_pattern_violations_by_hand_and_special_values():
    import oracle
    w = np.array([[1.0, 0.0, -2.0, 0.0], [0.0, -0.0, 3.0, 4.0]], dtype=np.float32)
    mask = np.array([[1, 1, 0, 0], [0, 0, 0, 1]], dtype=np.uint8)
    # removed and non-zero: (0,2) and (1,2); (0,3), (1,0) and (1,1) are removed zeros (-0 is a zero)
    assert oracle.pattern_violations(w, mask) == 2
    w[0, 3] = np.nan                                   # NaN is an active weight
    assert oracle.pattern_violations(w, mask) == 3
    assert oracle.pattern_violations(w, np.ones_like(mask)) == 0
    assert oracle.pattern_violations(w, np.zeros_like(mask)) == int(((w != 0) | np.isnan(w)).sum())
    bits = np.array([[0x3F80, 0x8000, 0x0000, 0x7FC0]], dtype=np.uint16)        # 1.0, -0, +0, NaN as bf16
    assert oracle.pattern_violations(bits, np.zeros((1, 4), dtype=np.uint8)) == 2


def test_groups_free_of_violations_follow_eq4():
    """Force N:M along rows on a tensor whose entries are zero with probability rho: a group of M loses no active
    weight iff it holds at least M - N zeros, which is the event whose probability Eq. 4 gives.  The observed
    share of violation-free groups must match it within sampling error (200000 groups: 5 sigma < 0.006)."""
    import oracle
    rng = np.random.default_rng(12)
    for N, M, rho in ((4, 8, 0.5), (2, 4, 0.7), (12, 16, 0.3)):
        w = rng.standard_normal((500, 400 * M)).astype(np.float32)
        w[rng.random(w.shape) < rho] = 0.0
        mask, _ = oracle.prune_1d(w, N, M)
        removed_active = ((w != 0) & (mask == 0)).reshape(500, 400, M).sum(-1)
        assert int(removed_active.sum()) == oracle.pattern_violations(w, mask)
        free = float((removed_active == 0).mean())
        want = float(oracle.nm_sparse_probability(M - N, M, rho))
        assert abs(free - want) < 0.006, (N, M, rho, free, want)

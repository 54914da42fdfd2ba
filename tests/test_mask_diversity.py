"""Mask diversity (Sec. 3, Eq. 2): the oracle's exact integer arithmetic against the values the paper prints in
Table 1, and the library's host routine against the oracle.  CPU only."""
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

"""Pins for the oracle's Algorithm 1 (CPU only).

Each test fixes the oracle against something that is not the oracle: the appendix's worked
example, the per-node K-lightest characterisation, hand-checkable 1:2 blocks, the Lemma with W*
from brute force, and symmetry invariants.
"""
import os

import numpy as np
import pytest

import oracle
from paper_2102_08124_amd import workloads as wl
from tests import refs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_tight_example():
    lines = [l for l in open(os.path.join(GOLDEN, "tight_example_4x4.txt")) if not l.startswith("#")]
    M, N = map(int, lines[0].split())
    blk = np.array([[float(x) for x in l.split()] for l in lines[1:1 + M]], dtype=np.float32)
    cnt, wp, wstar = map(float, lines[1 + M].split())
    return M, N, blk, int(cnt), wp, wstar


def test_tight_example_from_appendix():
    # App. A.2: seven unit edges are taken, the last one is u4->v4, optimum is the diagonal (4).
    M, N, blk, cnt, wp, wstar = _read_tight_example()
    mask, obj = oracle.approx(blk, N, M)
    pruned = 1 - mask
    assert pruned.sum() == cnt
    assert float((pruned * blk).sum()) == wp
    assert pruned[3, 3] == 1                              # u4 -> v4 is in P
    assert np.all(blk[pruned == 1] == 1.0)                # only unit edges were taken
    expect = np.zeros((4, 4), np.uint8)
    for i in range(4):
        expect[i, i] = 1
        if i:
            expect[i, i - 1] = 1
    assert np.array_equal(pruned, expect)
    assert obj == float(blk.sum()) - wp
    emask, eobj = oracle.exact(blk, N, M)
    assert float(blk.sum()) - eobj == wstar
    assert np.array_equal(1 - emask, np.eye(4, dtype=np.uint8))


@pytest.mark.parametrize("M", [2, 3, 5, 8, 16])
def test_tight_family_ratio(M):
    # Same construction at size M: ratio (2M-1)/M.
    blk = np.full((M, M), 10.0, np.float32)
    for i in range(M):
        blk[i, i] = 1.0
        if i:
            blk[i, i - 1] = 1.0
    mask, _ = oracle.approx(blk, M - 1, M)
    wp = float(((1 - mask) * blk).sum())
    assert wp == 2 * M - 1
    _, eobj = oracle.exact(blk, M - 1, M)
    assert float(blk.sum()) - eobj == M


def test_one_of_two_blocks_by_hand():
    # 1:2 -> a 2x2 block keeps (i,j) iff it is the larger of its row and the larger of its column.
    w = np.array([[1, 2, 5, 4],
                  [3, 4, 6, 7]], dtype=np.float32)
    mask, obj = oracle.approx(w, 1, 2)
    # block 0: rows keep {2},{4}; cols keep {3},{4} -> only 4 is kept.
    # block 1: rows keep {5},{7}; cols keep {6},{7} -> only 7.
    assert np.array_equal(mask, np.array([[0, 0, 0, 0], [0, 1, 0, 1]], np.uint8))
    assert obj == 11.0


def test_tie_break_is_row_major_index():
    # All magnitudes equal, 2:4 (K=2): the sweep visits (0,0),(0,1),... in row-major order.
    # Rows 0 and 1 are taken whole (row degree < 2 or column degree < 2 at every step), which
    # brings every column to degree 2; in rows 2 and 3 the first two entries are taken through
    # the row test, after which row and column are both saturated: the lower-right 2x2 survives.
    w = np.ones((4, 4), np.float32)
    mask, _ = oracle.approx(w, 2, 4)
    expect = np.zeros((4, 4), np.uint8)
    expect[2:, 2:] = 1
    assert np.array_equal(mask, expect)
    # Make (0,0) the single heaviest entry: it is visited last.  The sweep over the fifteen tied
    # entries goes as before except that row 0 now contributes only (0,1),(0,2),(0,3), so column 0
    # reaches degree 2 one row later; rows 2 and 3 again give up their first two entries and keep
    # (2,2),(2,3),(3,2),(3,3).  When (0,0) is reached row 0 has 3 and column 0 has 3: it is kept.
    w[0, 0] = 2.0
    mask, _ = oracle.approx(w, 2, 4)
    expect = np.zeros((4, 4), np.uint8)
    expect[2:, 2:] = 1
    expect[0, 0] = 1
    assert np.array_equal(mask, expect)


CASES = [(N, M) for M in (2, 4, 6, 8, 16) for N in range(1, M)] + [(N, 32) for N in (1, 5, 16, 20, 31)]


@pytest.mark.parametrize("N,M", CASES)
def test_matches_k_lightest_rule_random(N, M):
    rng = np.random.default_rng(100 * M + N)
    w = rng.standard_normal((4 * M, 6 * M)).astype(np.float32)
    mask, obj = oracle.approx(w, N, M)
    assert np.array_equal(mask, refs.k_lightest_rule(w, N, M))
    assert obj == pytest.approx(float((refs.magnitudes(w) * mask).sum()), rel=1e-12)


@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (3, 4), (4, 8), (8, 16), (3, 6), (16, 32), (7, 32)])
def test_matches_k_lightest_rule_ties_and_zeros(N, M):
    w = wl.tie_heavy_f32(8 * M, 8 * M, seed=7 + M, levels=4)
    mask, _ = oracle.approx(w, N, M)
    assert np.array_equal(mask, refs.k_lightest_rule(w, N, M))
    z = np.zeros((M, M), np.float32)
    mask, obj = oracle.approx(z, N, M)
    assert np.array_equal(mask, refs.k_lightest_rule(z, N, M)) and obj == 0.0


def test_bf16_and_special_values_use_bit_pattern_order():
    w = wl.special_values_f32(32, 32, seed=11)
    for N, M in ((2, 4), (4, 8)):
        mask, _ = oracle.approx(w, N, M)
        assert np.array_equal(mask, refs.k_lightest_rule(w, N, M))
    wb = wl.f32_to_bf16_bits(wl.gaussian_f32(64, 64, 12, std=0.02))
    for N, M in ((2, 4), (4, 8), (8, 16)):
        mask, obj = oracle.approx(wb, N, M)
        assert np.array_equal(mask, refs.k_lightest_rule(wb, N, M))
        assert obj == pytest.approx(float((refs.magnitudes(wb) * mask).sum()), rel=1e-12)
    # NaN is the heaviest magnitude, Inf next: in a 1:2 block they are what survives.
    blk = np.array([[np.nan, 1.0], [2.0, np.inf]], np.float32)
    mask, _ = oracle.approx(blk, 1, 2)
    assert np.array_equal(mask, np.array([[1, 0], [0, 1]], np.uint8))
    # -0 and +0 tie; denormals are not flushed (1e-45 > 0).
    blk = np.array([[-0.0, 0.0], [0.0, 1e-45]], np.float32)
    mask, _ = oracle.approx(blk, 1, 2)
    assert np.array_equal(mask, np.array([[0, 0], [0, 1]], np.uint8))


@pytest.mark.parametrize("N,M", [(2, 4), (4, 8), (8, 16), (1, 4), (3, 4), (2, 8)])
def test_cover_structure(N, M):
    # P is a cover: every row and column has >= K pruned, so the mask keeps <= N per row/column;
    # each pruned entry is among the K lightest of its row or of its column.
    K = M - N
    w = wl.gaussian_f32(8 * M, 8 * M, seed=21)
    mask, _ = oracle.approx(w, N, M)
    blocks = refs.to_blocks(mask, M)
    assert blocks.sum(axis=3).max() <= N and blocks.sum(axis=2).max() <= N
    assert (M - blocks.sum(axis=3)).min() >= K and (M - blocks.sum(axis=2)).min() >= K
    sc = oracle.score(w, mask, N, M)
    assert sc.row_violations == 0 and sc.col_violations == 0


def test_lemma_bound_with_brute_force_optimum():
    # Lemma (Sec. 4 / App. A.2): W(P) <= 2 W*, with W* from enumeration of Eq. 3's feasible set.
    for N, M in ((2, 4), (1, 4), (3, 4), (2, 5)):
        pats = refs.valid_patterns(N, M)
        for w in (wl.gaussian_f32(16 * M, 16 * M, seed=31), wl.tie_heavy_f32(16 * M, 16 * M, seed=32)):
            mask, _ = oracle.approx(w, N, M)
            a = refs.magnitudes(w)
            total = refs.per_block_sums(a, M)
            wp = total - refs.per_block_sums(a * mask, M)
            wstar = total - refs.brute_force_best(w, N, M, pats)
            assert np.all(wp <= 2.0 * wstar * (1 + 1e-9) + 1e-300)


def test_empirical_ratio_band():
    # Sec. 4.1 reports a pruned L1 about 1.2 times the optimum on trained nets;
    # on i.i.d. blocks the mean ratio lands close to that.
    w = wl.gaussian_f32(512, 512, seed=41)
    pats = refs.valid_patterns(2, 4)
    mask, _ = oracle.approx(w, 2, 4)
    a = refs.magnitudes(w)
    total = refs.per_block_sums(a, 4)
    ratio = (total - refs.per_block_sums(a * mask, 4)) / (total - refs.brute_force_best(w, 2, 4, pats))
    assert 1.1 < ratio.mean() < 1.35
    assert ratio.max() <= 2.0


@pytest.mark.parametrize("N,M", [(2, 4), (4, 8), (8, 16)])
def test_invariants(N, M):
    rng = np.random.default_rng(51 + M)
    w = rng.standard_normal((4 * M, 4 * M)).astype(np.float32)   # distinct magnitudes a.s.
    mask, _ = oracle.approx(w, N, M)
    signs = rng.integers(0, 2, w.shape).astype(np.float32) * 2 - 1
    assert np.array_equal(oracle.approx(w * signs, N, M)[0], mask)
    assert np.array_equal(oracle.approx(w * np.float32(0.125), N, M)[0], mask)
    assert np.array_equal(oracle.approx(np.ascontiguousarray(w.T), N, M)[0], mask.T)
    # permuting rows / columns inside each block permutes the mask the same way
    p, q = rng.permutation(M), rng.permutation(M)
    rows = (np.arange(w.shape[0]) // M) * M + p[np.arange(w.shape[0]) % M]
    cols = (np.arange(w.shape[1]) // M) * M + q[np.arange(w.shape[1]) % M]
    wp = np.ascontiguousarray(w[rows][:, cols])
    assert np.array_equal(oracle.approx(wp, N, M)[0], mask[rows][:, cols])


def test_threads_do_not_change_result():
    w = wl.gaussian_f32(64, 96, seed=61)
    m1, o1 = oracle.approx(w, 4, 8, threads=1)
    m4, o4 = oracle.approx(w, 4, 8, threads=4)
    assert np.array_equal(m1, m4) and o1 == pytest.approx(o4, rel=1e-14)


def test_shape_errors():
    w = np.zeros((6, 8), np.float32)
    with pytest.raises(ValueError):
        oracle.approx(w, 2, 4)
    with pytest.raises(ValueError):
        oracle.approx(np.zeros((8, 8), np.float32), 4, 4)
    with pytest.raises(ValueError):
        oracle.approx(np.zeros((8, 8), np.float32), 0, 4)


# ---- oracle.prune_1d: structured (non-transposable) N:M pruning along rows ----

def _prune_1d_numpy(w, N, M):
    """Independent statement with numpy: per group of M, stable argsort of the magnitude keys, keep the last N."""
    keys = refs.magnitude_keys(w) if hasattr(refs, "magnitude_keys") else None
    if keys is None:
        keys = (w.view(np.uint32) & 0x7FFFFFFF) if w.dtype == np.float32 else (w & 0x7FFF).astype(np.uint32)
    rows, cols = w.shape
    g = keys.reshape(rows, cols // M, M)
    order = np.argsort(g, axis=2, kind="stable")
    mask = np.zeros_like(g, dtype=np.uint8)
    np.put_along_axis(mask, order[:, :, M - N:], 1, axis=2)
    return mask.reshape(rows, cols)


@pytest.mark.parametrize("N,M", [(2, 4), (4, 8), (8, 16), (1, 4), (3, 4), (5, 8), (1, 2)])
def test_prune_1d_matches_numpy_statement(N, M):
    for w in (wl.gaussian_f32(6, 16 * M, seed=900 + M), wl.tie_heavy_f32(8, 8 * M, seed=901 + N),
              wl.special_values_f32(4, 16 * M, seed=902), wl.f32_to_bf16_bits(wl.gaussian_f32(8, 8 * M, seed=903, std=0.02))):
        mask, obj = oracle.prune_1d(w, N, M)
        want = _prune_1d_numpy(w, N, M)
        assert np.array_equal(mask, want)
        assert (mask.reshape(w.shape[0], -1, M).sum(axis=2) == N).all()        # exactly N kept per group
        a = refs.magnitudes(w)
        with np.errstate(invalid="ignore"):
            kept = float((a * mask).sum())
        assert (np.isnan(obj) and np.isnan(kept)) or obj == pytest.approx(kept, rel=1e-12)


def test_prune_1d_hand_example_and_relation_to_transposable():
    w = np.array([[0.1, -0.4, 0.3, 0.4, 0.0, -0.0, 0.0, 1.0]], dtype=np.float32)
    mask, obj = oracle.prune_1d(w, 2, 4)
    # group 1: |.| = .1 .4 .3 .4 -> keep the two 0.4 (positions 1, 3); group 2: ties at zero -> later position kept
    assert mask.tolist() == [[0, 1, 0, 1, 0, 0, 1, 1]]
    assert obj == pytest.approx(0.4 + 0.4 + 1.0, rel=1e-6)
    # row-only pruning keeps at least as much L1 as any transposable mask (it is a relaxation of Eq. 3)
    wb = wl.gaussian_f32(32, 32, seed=910)
    _, obj1 = oracle.prune_1d(wb, 2, 4)
    _, obj_t = oracle.exact(wb, 2, 4)
    assert obj1 >= obj_t * (1 - 1e-12)

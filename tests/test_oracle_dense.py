"""Pins of the oracle's dense masked copy and mean absorption (Sec. 4; Sec. 5, bias fix)."""
import numpy as np
import pytest

import oracle


def test_hand_computed_groups():
    # group (1, -2, 3, 4), kept first and last: pruned mean (-2 + 3)/2 = 0.5
    w = np.array([[1.0, -2.0, 3.0, 4.0, 1.0, 2.0, 3.0, -4.0]])
    m = np.array([[1, 0, 0, 1, 1, 1, 1, 0]], dtype=np.uint8)
    np.testing.assert_array_equal(oracle.apply_dense(w, m), [[1, 0, 0, 4, 1, 2, 3, 0]])
    # second group prunes one weight of four: its mean is the weight itself, every kept one receives it
    np.testing.assert_array_equal(oracle.apply_dense(w, m, 4, True), [[1.5, 0, 0, 4.5, -3, -2, -1, 0]])


def test_groups_with_nothing_pruned_or_nothing_kept():
    w = np.array([[1.0, 2.0, 3.0, 4.0, 5.0, 6.0, 7.0, 8.0]])
    m = np.array([[1, 1, 1, 1, 0, 0, 0, 0]], dtype=np.uint8)
    np.testing.assert_array_equal(oracle.apply_dense(w, m, 4, True), [[1, 2, 3, 4, 0, 0, 0, 0]])


@pytest.mark.parametrize("N,M", [(2, 4), (4, 8), (8, 16)])
def test_half_sparsity_keeps_every_group_sum(N, M):
    # with as many kept as pruned weights per group, adding the pruned mean to each kept weight moves exactly the
    # pruned sum onto the kept ones: the group's sum, hence the row's response to a constant input, is unchanged
    rng = np.random.default_rng(5)
    w = rng.standard_normal((32, 8 * M))
    mask, _ = oracle.prune_1d(w.astype(np.float32), N, M)
    w = w.astype(np.float32).astype(np.float64)
    out = oracle.apply_dense(w, mask, M, True)
    np.testing.assert_allclose(out.reshape(32, 8, M).sum(-1), w.reshape(32, 8, M).sum(-1), rtol=0, atol=1e-12)
    assert ((out != 0) <= (mask != 0)).all()
    # and without absorption the sums differ by the pruned mass
    plain = oracle.apply_dense(w, mask)
    np.testing.assert_array_equal(plain, w * mask)


def test_transposable_mask_rows_are_the_groups():
    # the groups run along rows: transposing both operands gives a different result unless the mask is symmetric
    rng = np.random.default_rng(6)
    w = rng.standard_normal((8, 8)).astype(np.float32)
    mask, _ = oracle.approx(w, 2, 4)
    a = oracle.apply_dense(w, mask, 4, True)
    for r in range(8):
        for g in (0, 4):
            k = mask[r, g:g + 4] != 0
            if 0 < k.sum() < 4:
                want = w[r, g:g + 4].astype(np.float64)[k] + w[r, g:g + 4].astype(np.float64)[~k].mean()
                np.testing.assert_allclose(a[r, g:g + 4][k], want, rtol=1e-15)

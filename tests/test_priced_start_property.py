"""The property the exact solver's start relies on (successive shortest augmenting paths need a start that is
cheapest for its own row counts): if every column prunes the K entries with the smallest cost + price(row), then
among all prunings with K entries per column and the same number of entries per row, this one has the least total
cost -- whatever the prices.  Checked here by enumeration on small blocks; plain numpy, no GPU, no oracle."""
import itertools

import numpy as np
import pytest


def _greedy(cost, price, K):
    M = cost.shape[0]
    x = np.zeros((M, M), dtype=np.int64)
    key = (cost + price[:, None]) * M + np.arange(M)[:, None]        # ties: lower row first
    for j in range(M):
        x[np.argsort(key[:, j], kind="stable")[:K], j] = 1
    return x


@pytest.mark.parametrize("M,K", [(4, 2), (4, 1), (5, 2)])
def test_column_greedy_under_row_prices_is_cheapest_for_its_row_counts(M, K):
    rng = np.random.default_rng(70 + M + K)
    col_patterns = [np.array(p) for p in itertools.product((0, 1), repeat=M) if sum(p) == K]
    for trial in range(12):
        cost = rng.integers(0, 50, size=(M, M))                      # small range: ties on purpose
        price = rng.integers(-40, 40, size=M)
        x = _greedy(cost, price, K)
        rows = x.sum(axis=1)
        assert np.all(x.sum(axis=0) == K)
        best = None
        for combo in itertools.product(col_patterns, repeat=M):
            y = np.stack(combo, axis=1)
            if np.array_equal(y.sum(axis=1), rows):
                c = int((cost * y).sum())
                best = c if best is None else min(best, c)
        assert int((cost * x).sum()) == best


def test_prices_that_follow_the_imbalance_reduce_it():
    # the rounds the kernel runs: price += step * (count - K), step shrinking; the excess left never grows when the
    # best round is kept, and on random blocks it falls well below the unpriced start's
    rng = np.random.default_rng(77)
    M, K = 8, 4
    before = after = 0
    for trial in range(200):
        cost = np.abs(rng.standard_normal((M, M)) * 1e6).astype(np.int64)
        price = np.zeros(M, dtype=np.int64)
        x = _greedy(cost, price, K)
        e0 = best = int(np.maximum(x.sum(axis=1) - K, 0).sum())
        step = 3 * int(cost.max()) // 64
        for r in range(10):
            price = price + step * (x.sum(axis=1) - K)
            step = step * 11 // 16
            x = _greedy(cost, price, K)
            best = min(best, int(np.maximum(x.sum(axis=1) - K, 0).sum()))
        before += e0
        after += best
    assert after * 4 < before

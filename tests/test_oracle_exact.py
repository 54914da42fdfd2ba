"""Pins for the oracle's exact solver (Eq. 3 through the Fig. 3 min-cost flow), CPU only."""
import numpy as np
import pytest

import oracle
from paper_2102_08124_amd import workloads as wl
from tests import refs


def test_pattern_counts():
    # 0/1 matrices with all row and column sums N: 90 for 4x4 with N=2; M! for N=1.
    assert len(refs.valid_patterns(2, 4)) == 90
    assert len(refs.valid_patterns(1, 4)) == 24
    assert len(refs.valid_patterns(1, 3)) == 6
    assert len(refs.valid_patterns(2, 5)) == 2040


def test_network_sizes_match_fig3():
    # App. A.3: 2M+2 nodes, M^2+2M edges, flow demand M*K (= M^2/2 when K = M/2).
    for N, M in ((2, 4), (4, 8), (8, 16), (1, 4), (6, 8)):
        assert oracle.network_sizes(N, M) == (2 * M + 2, M * M + 2 * M, M * (M - N))


def _check_exact_mask(w, mask, obj, per_block, N, M):
    blocks = refs.to_blocks(mask, M)
    assert np.all(blocks.sum(axis=3) == N) and np.all(blocks.sum(axis=2) == N)
    kept = refs.per_block_sums(refs.magnitudes(w) * mask, M)
    np.testing.assert_allclose(per_block, kept, rtol=1e-13, atol=0)
    assert obj == pytest.approx(float(kept.sum()), rel=1e-12)


@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (3, 4), (1, 2), (1, 3), (2, 3), (2, 5), (3, 5)])
def test_equals_brute_force(N, M):
    pats = refs.valid_patterns(N, M)
    for w in (wl.gaussian_f32(16 * M, 16 * M, seed=200 + M), wl.laplace_f32(8 * M, 8 * M, seed=201 + N),
              wl.tie_heavy_f32(8 * M, 8 * M, seed=202)):
        mask, obj, pb = oracle.exact(w, N, M, per_block=True)
        _check_exact_mask(w, mask, obj, pb, N, M)
        np.testing.assert_allclose(pb, refs.brute_force_best(w, N, M, pats), rtol=1e-12, atol=1e-300)


def test_config1_exact_equals_90_pattern_enumeration():
    w = wl.config1()
    mask, obj, pb = oracle.exact(w, 2, 4, per_block=True)
    _check_exact_mask(w, mask, obj, pb, 2, 4)
    best = refs.brute_force_best(w, 2, 4)
    assert best.shape == (16, 16)
    np.testing.assert_allclose(pb, best, rtol=1e-13)


@pytest.mark.parametrize("N,M", [(4, 8), (8, 16), (3, 8), (5, 8), (2, 6), (16, 32), (9, 32)])
def test_equals_lp_optimum(N, M):
    for k, w in enumerate((wl.gaussian_f32(2 * M, 3 * M, seed=210 + M), wl.laplace_f32(2 * M, 2 * M, seed=211),
                           wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(wl.gaussian_f32(2 * M, 2 * M, 212, std=0.02))))):
        mask, obj, pb = oracle.exact(w, N, M, per_block=True)
        _check_exact_mask(w, mask, obj, pb, N, M)
        a = refs.to_blocks(refs.magnitudes(w), M)
        for br in range(a.shape[0]):
            for bc in range(a.shape[1]):
                assert pb[br, bc] == pytest.approx(refs.lp_best(a[br, bc], N), rel=1e-9, abs=1e-12)


@pytest.mark.parametrize("M", [4, 8, 16])
def test_assignment_special_cases(M):
    from scipy.optimize import linear_sum_assignment
    w = wl.laplace_f32(4 * M, 4 * M, seed=220 + M)
    a = refs.to_blocks(refs.magnitudes(w), M)
    # N = 1: keep a maximum-weight perfect matching.
    _, _, pb1 = oracle.exact(w, 1, M, per_block=True)
    # N = M-1: prune a minimum-weight perfect matching.
    _, _, pbm = oracle.exact(w, M - 1, M, per_block=True)
    for br in range(a.shape[0]):
        for bc in range(a.shape[1]):
            blk = a[br, bc]
            r, c = linear_sum_assignment(blk, maximize=True)
            assert pb1[br, bc] == pytest.approx(blk[r, c].sum(), rel=1e-12)
            r, c = linear_sum_assignment(blk)
            assert pbm[br, bc] == pytest.approx(blk.sum() - blk[r, c].sum(), rel=1e-12)


def test_third_opinion_network_simplex():
    import networkx as nx
    M, N = 8, 4
    K = M - N
    rng = np.random.default_rng(230)
    w = rng.integers(0, 1000, size=(2 * M, 2 * M)).astype(np.float32)
    _, _, pb = oracle.exact(w, N, M, per_block=True)
    a = refs.to_blocks(refs.magnitudes(w), M)
    for br in range(2):
        for bc in range(2):
            g = nx.DiGraph()
            g.add_node("s", demand=-M * K)
            g.add_node("t", demand=M * K)
            for i in range(M):
                g.add_edge("s", ("r", i), capacity=K, weight=0)
                g.add_edge(("c", i), "t", capacity=K, weight=0)
                for j in range(M):
                    g.add_edge(("r", i), ("c", j), capacity=1, weight=int(a[br, bc, i, j]))
            cost = nx.min_cost_flow_cost(g)
            assert pb[br, bc] == a[br, bc].sum() - cost


@pytest.mark.parametrize("N,M", [(2, 4), (4, 8), (8, 16)])
def test_invariants(N, M):
    rng = np.random.default_rng(240 + M)
    w = rng.standard_normal((3 * M, 3 * M)).astype(np.float32)
    mask, obj, pb = oracle.exact(w, N, M, per_block=True)
    a = refs.magnitudes(w)
    signs = rng.integers(0, 2, w.shape).astype(np.float32) * 2 - 1
    assert np.array_equal(oracle.exact(w * signs, N, M)[0], mask)
    m2, o2 = oracle.exact(w * np.float32(4.0), N, M)
    assert o2 == pytest.approx(4.0 * obj, rel=1e-13)
    mt, ot, pbt = oracle.exact(np.ascontiguousarray(w.T), N, M, per_block=True)
    np.testing.assert_allclose(pbt, pb.T, rtol=1e-13)
    p, q = rng.permutation(M), rng.permutation(M)
    rows = (np.arange(w.shape[0]) // M) * M + p[np.arange(w.shape[0]) % M]
    cols = (np.arange(w.shape[1]) // M) * M + q[np.arange(w.shape[1]) % M]
    _, _, pbp = oracle.exact(np.ascontiguousarray(w[rows][:, cols]), N, M, per_block=True)
    np.testing.assert_allclose(pbp, pb, rtol=1e-13)
    # pruned weight is at least the K lightest of every row (and of every column)
    K = M - N
    blocks = refs.to_blocks(a, M)
    total = blocks.sum(axis=(2, 3))
    low_r = np.sort(blocks, axis=3)[..., :K].sum(axis=(2, 3))
    low_c = np.sort(blocks, axis=2)[:, :, :K, :].sum(axis=(2, 3))
    assert np.all(total - pb >= np.maximum(low_r, low_c) * (1 - 1e-12))
    # complement symmetry for N = M/2: keeping the best N-regular set prunes the lightest one
    neg = (a.max() + 1.0 - a).astype(np.float32)          # reverses the order of magnitudes
    if N == K:
        _, _, pbn = oracle.exact(neg, N, M, per_block=True)
        negblocks = refs.to_blocks(refs.magnitudes(neg), M).sum(axis=(2, 3))
        # min pruned of neg  <->  max kept of w (up to the float32 rounding of `neg`)
        np.testing.assert_allclose(negblocks - pbn, N * M * (a.max() + 1.0) - pb, rtol=1e-5)


def test_approx_can_beat_exact_on_retained_l1():
    # The greedy cover may prune more than K per row/column cheaply, so its retained L1 can exceed
    # the equality-constrained optimum; only the pruned-weight bound W(P) <= 2W* is guaranteed.
    blk = np.full((4, 4), 1e-3, np.float32)
    for (i, j) in ((0, 0), (0, 1), (1, 1), (1, 2), (2, 2), (2, 0)):
        blk[i, j] = 1.0
    am, aobj = oracle.approx(blk, 2, 4)
    em, eobj = oracle.exact(blk, 2, 4)
    # greedy keeps the six heavy entries plus (3,3), which is outside the 2 lightest of its row and column
    assert aobj == pytest.approx(6.001, rel=1e-6) and am.sum() == 7
    assert eobj < aobj
    assert eobj == pytest.approx(refs.brute_force_best(blk, 2, 4)[0, 0], rel=1e-12)


def test_threads_do_not_change_result():
    w = wl.laplace_f32(64, 64, seed=250)
    m1, o1, p1 = oracle.exact(w, 4, 8, threads=1, per_block=True)
    m3, o3, p3 = oracle.exact(w, 4, 8, threads=3, per_block=True)
    assert np.array_equal(p1, p3) and o1 == pytest.approx(o3, rel=1e-14)

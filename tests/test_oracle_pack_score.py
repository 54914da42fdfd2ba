"""Pins for the oracle's score and apply+pack (CPU only)."""
import os

import numpy as np
import pytest

import oracle
from oracle.oracle import index_bits, packed_shapes
from paper_2102_08124_amd import workloads as wl
from tests import refs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_score_matches_definitions():
    for N, M in ((2, 4), (4, 8), (8, 16)):
        w = wl.gaussian_f32(4 * M, 8 * M, seed=300 + M)
        rng = np.random.default_rng(301)
        mask = (rng.random(w.shape) < 0.5).astype(np.uint8)
        sc = oracle.score(w, mask, N, M)
        a = refs.magnitudes(w)
        assert sc.retained_l1 == pytest.approx(float((a * mask).sum()), rel=1e-12)
        assert sc.total_l1 == pytest.approx(float(a.sum()), rel=1e-12)
        assert sc.kept == int(mask.sum())
        b = refs.to_blocks(mask, M)
        assert sc.row_violations == int((b.sum(axis=3) > N).sum())
        assert sc.col_violations == int((b.sum(axis=2) > N).sum())
        assert sc.row_not_n == int((b.sum(axis=3) != N).sum())
        assert sc.col_not_n == int((b.sum(axis=2) != N).sum())
        np.testing.assert_allclose(sc.per_block, refs.per_block_sums(a * mask, M), rtol=1e-13)


def test_pack_hand_example():
    rows = {}
    for line in open(os.path.join(GOLDEN, "pack_example_2of4.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        rows[k] = v
    w = np.array([rows["w"]], dtype=np.float32)
    w = np.vstack([w, np.zeros((3, 8), np.float32)])                # pad to 4 rows (M = 4)
    mask = np.zeros((4, 8), np.uint8)
    mask[0] = np.array(rows["mask"], dtype=np.uint8)
    vals, idx, valsT, idxT = oracle.apply_pack(w, mask, 2, 4)
    assert vals.shape == (4, 4) and idx.shape == (4, 1)
    assert np.array_equal(vals[0], np.array(rows["vals"], dtype=np.float32))
    assert not np.signbit(vals[0, 2])                               # filler is +0
    assert idx[0, 0] == int(rows["idx"][0])


def _roundtrip(w, mask, N, M):
    rows, cols = w.shape
    vals, idx, valsT, idxT = oracle.apply_pack(w, mask, N, M)
    shp = packed_shapes(rows, cols, N, M)
    assert (vals.shape, idx.shape, valsT.shape, idxT.shape) == shp
    masked = np.where(mask != 0, w, np.zeros_like(w))
    assert np.array_equal(oracle.unpack(vals, idx, rows, cols, N, M).view(np.uint8), masked.view(np.uint8))
    assert np.array_equal(oracle.unpack(valsT, idxT, cols, rows, N, M).view(np.uint8),
                          np.ascontiguousarray(masked.T).view(np.uint8))
    ib = index_bits(M)
    for r in (0, rows - 1):
        p = refs.unpack_indices(idx[r], cols // M * N, ib).reshape(-1, N)
        assert np.all(np.diff(p, axis=1) > 0) and p.max() < M
    for r in (0, cols - 1):
        p = refs.unpack_indices(idxT[r], rows // M * N, ib).reshape(-1, N)
        assert np.all(np.diff(p, axis=1) > 0) and p.max() < M
    return vals, valsT


@pytest.mark.parametrize("N,M", [(2, 4), (4, 8), (8, 16), (1, 4), (3, 8), (16, 32), (5, 32)])
def test_pack_roundtrip_exact_and_approx_masks(N, M):
    w = wl.gaussian_f32(4 * M, 6 * M, seed=310 + M)
    w[0, 0] = -0.0
    for mask, obj in (oracle.exact(w, N, M), oracle.approx(w, N, M)):   # approx: fewer than N kept in places
        vals, valsT = _roundtrip(w, mask, N, M)
        assert np.abs(vals.astype(np.float64)).sum() == pytest.approx(obj, rel=1e-12)
        assert np.abs(valsT.astype(np.float64)).sum() == pytest.approx(obj, rel=1e-12)


def test_pack_bf16_and_non_finite():
    wb = wl.f32_to_bf16_bits(wl.gaussian_f32(16, 32, seed=320, std=0.02))
    mask, _ = oracle.approx(wb, 2, 4)
    _roundtrip(wb, mask, 2, 4)
    w = wl.special_values_f32(16, 16, seed=321)
    mask, _ = oracle.approx(w, 2, 4)
    _roundtrip(w, mask, 2, 4)      # pruned NaN/Inf become +0 (select, not multiply)


def test_empty_mask_packs_fillers_only():
    w = wl.gaussian_f32(8, 8, seed=330)
    vals, idx, valsT, idxT = oracle.apply_pack(w, np.zeros((8, 8), np.uint8), 2, 4)
    assert not vals.any() and not valsT.any()
    # fillers take positions 0 and 1 of each group: slots (0,1) -> bits 00,01 -> nibble 0b0100
    assert np.all(idx == 0x44) and np.all(idxT == 0x44)


# ---- oracle.spmm: products with the packed operands (forward W, backward W^T) ----

def _spmm_case(seed, rows=16, cols=64, tokens=5):
    w = wl.f32_to_bf16_bits(wl.gaussian_f32(rows, cols, seed, std=0.5))
    mask, _ = oracle.exact(w, 2, 4)
    x = wl.f32_to_bf16_bits(wl.gaussian_f32(tokens, cols, seed + 1))
    g = wl.f32_to_bf16_bits(wl.gaussian_f32(tokens, rows, seed + 2))
    return w, mask, x, g


def test_spmm_matches_pure_python_loops():
    # brute force with Python floats (doubles), no numpy product, on a tiny case
    w, mask, x, g = _spmm_case(700, rows=8, cols=8, tokens=3)
    vals, idx, valsT, idxT = oracle.apply_pack(w, mask, 2, 4)
    wf, xf, gf = oracle.bf16_to_f64(w), oracle.bf16_to_f64(x), oracle.bf16_to_f64(g)
    fwd = oracle.spmm(vals, idx, 8, 8, 2, 4, x)
    bwd = oracle.spmm(valsT, idxT, 8, 8, 2, 4, g)
    for t in range(3):
        for r in range(8):
            acc = 0.0
            for c in range(8):
                if mask[r, c]:
                    acc += float(xf[t, c]) * float(wf[r, c])
            assert fwd[t, r] == pytest.approx(acc, rel=1e-14, abs=1e-300)
        for c in range(8):
            acc = 0.0
            for r in range(8):
                if mask[r, c]:
                    acc += float(gf[t, r]) * float(wf[r, c])       # (W^T g)_c = sum_r W[r][c] g[r]
            assert bwd[t, c] == pytest.approx(acc, rel=1e-14, abs=1e-300)


def test_spmm_identity_and_linearity():
    w, mask, x, g = _spmm_case(710)
    vals, idx, valsT, idxT = oracle.apply_pack(w, mask, 2, 4)
    masked = np.where(mask != 0, oracle.bf16_to_f64(w), 0.0)
    eye_in = np.eye(64, dtype=np.float32)
    assert np.array_equal(oracle.spmm(vals, idx, 16, 64, 2, 4, eye_in), masked.T)       # x = I  ->  y = Wd^T
    eye_out = np.eye(16, dtype=np.float32)
    assert np.array_equal(oracle.spmm(valsT, idxT, 64, 16, 2, 4, eye_out), masked)     # backward with g = I -> Wd
    xf = oracle.bf16_to_f64(x)
    y = oracle.spmm(vals, idx, 16, 64, 2, 4, x)
    y2 = oracle.spmm(vals, idx, 16, 64, 2, 4, (2.0 * xf).astype(np.float32))
    np.testing.assert_allclose(y2, 2.0 * y, rtol=1e-14)
    # <W x, g> = <x, W^T g>: forward and backward operands describe the same matrix
    gf = oracle.bf16_to_f64(g)
    lhs = float((y * gf).sum())
    rhs = float((xf * oracle.spmm(valsT, idxT, 64, 16, 2, 4, g)).sum())
    assert lhs == pytest.approx(rhs, rel=1e-12)


# ---- flip_count: the number of entries whose kept / pruned state differs (Sec. 4.1: the mask is re-extracted as the
# weights move; the flip fraction is this count over rows * cols).  Pinned by hand-counted masks, not by its own formula.

def test_flip_count_hand_counted():
    # kept = any non-zero byte.  Positions that differ in STATE, counted by hand: (0,1) kept->pruned, (0,3) pruned->kept,
    # (1,0) pruned->kept, (2,2) kept->pruned = 4.  (0,0) 1 vs 255 and (1,3) 7 vs 1 differ as bytes but not in state.
    a = np.array([[1, 9, 0, 0],
                  [0, 0, 1, 7],
                  [0, 1, 200, 0]], dtype=np.uint8)
    b = np.array([[255, 0, 0, 3],
                  [1, 0, 1, 1],
                  [0, 1, 0, 0]], dtype=np.uint8)
    assert oracle.flip_count(a, b) == 4
    assert oracle.flip_count(b, a) == 4                       # symmetric
    assert oracle.flip_count(a, a) == 0                       # identical masks
    assert oracle.flip_count(a, (a != 0).astype(np.uint8)) == 0   # byte values do not matter, only kept / pruned
    # byte equality would have said 6 here: the two same-state pairs with different bytes must not count
    assert int((a != b).sum()) == 6


def test_flip_count_all_flipped_and_brute_force():
    rng = np.random.default_rng(77)
    a = (rng.random((13, 40)) < 0.4).astype(np.uint8)
    assert oracle.flip_count(a, 1 - a) == a.size              # every entry changes state
    assert oracle.flip_count(np.zeros_like(a), a) == int(a.sum())
    b = (rng.random((13, 40)) < 0.6).astype(np.uint8) * rng.integers(1, 256, size=(13, 40)).astype(np.uint8)
    n = 0
    for i in range(13):                                       # plain loops over the definition
        for j in range(40):
            ka, kb = a[i, j] != 0, b[i, j] != 0
            n += 1 if (ka and not kb) or (kb and not ka) else 0
    assert oracle.flip_count(a, b) == n
    # triangle inequality and additivity over a partition of the entries
    c = (rng.random((13, 40)) < 0.5).astype(np.uint8)
    assert oracle.flip_count(a, c) <= oracle.flip_count(a, b) + oracle.flip_count(b, c)
    assert oracle.flip_count(a, b) == oracle.flip_count(a[:, :24], b[:, :24]) + oracle.flip_count(a[:, 24:], b[:, 24:])


def test_flip_count_strided_view_and_bit_masks():
    rng = np.random.default_rng(78)
    big_a = (rng.random((9, 64)) < 0.5).astype(np.uint8)
    big_b = (rng.random((9, 80)) < 0.5).astype(np.uint8)
    a, b = big_a[:, 8:40], big_b[:, 16:48]                    # column slices: row stride > cols
    want = sum(int(bool(a[i, j]) != bool(b[i, j])) for i in range(9) for j in range(32))
    assert oracle.flip_count(a, b) == want
    # BITS masks (bit c % 8 of byte c / 8, LSB first): popcount of the xor of the packed bytes is the same count
    pa = np.packbits(a, axis=1, bitorder="little")
    pb = np.packbits(b, axis=1, bitorder="little")
    assert pa[0, 0] & 1 == a[0, 0] and (pa[0, 0] >> 3) & 1 == a[0, 3]          # LSB-first layout
    xor_pop = sum(bin(int(x)).count("1") for x in (pa ^ pb).ravel())
    assert xor_pop == want
    ua = np.unpackbits(pa, axis=1, bitorder="little")[:, :32]
    ub = np.unpackbits(pb, axis=1, bitorder="little")[:, :32]
    assert oracle.flip_count(ua, ub) == want

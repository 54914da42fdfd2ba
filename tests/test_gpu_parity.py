"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bars: approximation masks bit-exact; exact-solver masks valid (exactly N per row/column) with every
block's retained L1 equal to the oracle's within 1e-5 relative; objectives within 1e-5 relative
(fp32 per strip, fp64 across strips on the GPU; fp64 in the oracle).
"""
import numpy as np
import pytest

import oracle
from paper_2102_08124_amd import workloads as wl
from tests import refs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2102_08124_amd import binding as tm   # noqa: E402
from tests.gpu_util import run_masks, run_score  # noqa: E402

NM = [(2, 4), (4, 8), (8, 16)]
FMTS = [tm.TMASK_MASK_U8, tm.TMASK_MASK_BITS]


def _inputs(kind, rows, cols, seed):
    if kind == "f32":
        return wl.gaussian_f32(rows, cols, seed)
    if kind == "bf16":
        return wl.f32_to_bf16_bits(wl.gaussian_f32(rows, cols, seed, std=0.02))
    if kind == "ties":
        return wl.tie_heavy_f32(rows, cols, seed, levels=4)
    if kind == "ties_bf16":
        return wl.f32_to_bf16_bits(wl.tie_heavy_f32(rows, cols, seed, levels=3))
    if kind == "special":
        return wl.special_values_f32(rows, cols, seed)
    raise ValueError(kind)


def _check_exact(w, mask, N, M, oracle_pb):
    b = refs.to_blocks(mask, M)
    assert np.all(b.sum(axis=3) == N) and np.all(b.sum(axis=2) == N), "mask is not exactly N per row/column"
    got = refs.per_block_sums(refs.magnitudes(w) * mask, M)
    np.testing.assert_allclose(got, oracle_pb, rtol=1e-5, atol=1e-30)


# ---------------------------------------------------------------- approximation ----------------

@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("N,M", NM)
@pytest.mark.parametrize("kind", ["f32", "bf16", "ties", "ties_bf16", "special"])
def test_approx_bit_exact_ragged(kind, N, M, fmt):
    # 5 block-rows x 1008 columns: several 256-strip tiles and a ragged last tile
    w = _inputs(kind, 5 * M, 1008, seed=1000 + M)
    (mask,), obj = run_masks(tm.tmask_approx, [w], N, M, fmt)
    omask, oobj = oracle.approx(w, N, M)
    assert np.array_equal(mask, omask)
    if kind != "special":
        assert obj[0] == pytest.approx(oobj, rel=1e-5)


@pytest.mark.parametrize("N,M", [(1, 4), (3, 4), (1, 8), (2, 8), (3, 8), (5, 8), (6, 8), (7, 8), (1, 16), (3, 16), (5, 16), (12, 16),
                                 (15, 16)])
def test_approx_other_n(N, M):
    # "ties": the threshold forms for any N at M = 8 must notice cuts among equal values (fp32) or settle them by
    # position (bf16)
    for kind in ("f32", "bf16", "ties", "ties_bf16"):
        w = _inputs(kind, 3 * M, 512, seed=1100 + N)
        (mask,), obj = run_masks(tm.tmask_approx, [w], N, M)
        omask, oobj = oracle.approx(w, N, M)
        assert np.array_equal(mask, omask)
        assert obj[0] == pytest.approx(oobj, rel=1e-5)


@pytest.mark.parametrize("N,M", NM)
@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_approx_sparse_ties_inside_random_data(dt, N, M):
    # mostly distinct magnitudes with a few tied lines: the fp32 threshold kernels must notice a tie across the
    # cut in single lanes of a wavefront and fall back to the rank form there
    w = wl.gaussian_f32(4 * M, 1024, seed=1500 + M)
    rng = np.random.default_rng(1501)
    for _ in range(40):
        r, c = int(rng.integers(0, w.shape[0])), int(rng.integers(0, w.shape[1] - M))
        w[r, c:c + M] = np.float32(0.5) * np.sign(w[r, c:c + M] + np.float32(1e-9))      # one tied row segment
    for _ in range(40):
        r, c = int(rng.integers(0, w.shape[0] - M)), int(rng.integers(0, w.shape[1]))
        w[r:r + M, c] = 0.0                                                               # one zero column segment
    if dt == "bf16":
        w = wl.f32_to_bf16_bits(w)
    (mask,), obj = run_masks(tm.tmask_approx, [w], N, M)
    omask, oobj = oracle.approx(w, N, M)
    assert np.array_equal(mask, omask)
    assert obj[0] == pytest.approx(oobj, rel=1e-5)


def test_approx_config1():
    w = wl.config1()
    (mask,), obj = run_masks(tm.tmask_approx, [w], 2, 4)
    omask, oobj = oracle.approx(w, 2, 4)
    assert np.array_equal(mask, omask) and obj[0] == pytest.approx(oobj, rel=1e-6)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_approx_batched_many_matrices_and_strides(dt):
    # 70 matrices (> one 64-matrix launch), mixed shapes incl. the smallest legal ones, ld > cols
    rng = np.random.default_rng(5)
    shapes = [(16, 16), (16, 32), (32, 16), (64, 48), (16, 1040), (128, 272)]
    ws = [_inputs(dt, *shapes[int(rng.integers(len(shapes)))], seed=1200 + k) for k in range(70)]
    for N, M in NM:
        masks, obj = run_masks(tm.tmask_approx, ws, N, M, ld_pad=32)
        for k, w in enumerate(ws):
            omask, oobj = oracle.approx(w, N, M)
            assert np.array_equal(masks[k], omask), "matrix %d" % k
            assert obj[k] == pytest.approx(oobj, rel=1e-5)


def test_approx_without_objective_or_workspace():
    w = _inputs("f32", 32, 64, seed=1300)
    wd = torch.from_numpy(w).cuda()
    masks = tm.alloc_masks([wd])
    tm.tmask_approx([wd], masks, 2, 4)            # no objective -> no workspace needed
    torch.cuda.synchronize()
    assert np.array_equal(masks[0].cpu().numpy(), oracle.approx(w, 2, 4)[0])


# ---------------------------------------------------------------- exact ------------------------

@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("N,M", NM)
@pytest.mark.parametrize("kind", ["f32", "bf16", "ties", "ties_bf16"])
def test_exact_optimal_ragged(kind, N, M, fmt):
    w = _inputs(kind, 5 * M, 1008, seed=2000 + M)
    (mask,), obj = run_masks(tm.tmask_exact, [w], N, M, fmt)
    _, oobj, opb = oracle.exact(w, N, M, per_block=True, threads=8)
    _check_exact(w, mask, N, M, opb)
    assert obj[0] == pytest.approx(oobj, rel=1e-5)


def test_exact_config1_against_enumeration():
    w = wl.config1()
    (mask,), obj = run_masks(tm.tmask_exact, [w], 2, 4)
    best = refs.brute_force_best(w, 2, 4)          # all 90 patterns per block
    _check_exact(w, mask, 2, 4, best)
    _, oobj, opb = oracle.exact(w, 2, 4, per_block=True)
    np.testing.assert_allclose(opb, best, rtol=1e-12)
    assert obj[0] == pytest.approx(oobj, rel=1e-6)


@pytest.mark.parametrize("N,M", [(1, 4), (3, 4), (2, 8), (6, 8), (1, 8), (7, 8), (4, 16), (12, 16), (15, 16)])
def test_exact_other_n(N, M):
    for kind in ("f32", "bf16"):
        w = _inputs(kind, 2 * M, 528, seed=2100 + N)
        (mask,), obj = run_masks(tm.tmask_exact, [w], N, M)
        _, oobj, opb = oracle.exact(w, N, M, per_block=True, threads=8)
        _check_exact(w, mask, N, M, opb)


@pytest.mark.parametrize("N,M", NM)
def test_exact_heavy_tailed_and_degenerate(N, M):
    w = wl.laplace_f32(4 * M, 512, seed=2200 + M)
    w[:M, :M] = 0.0                                   # an all-zero block
    w[M:2 * M, :M] = 1.0                              # an all-equal block
    w[:M, M:2 * M] = np.float32(1e-30)                # tiny magnitudes
    w[M:2 * M, M:2 * M] *= np.float32(1e30)           # huge magnitudes
    w[0, 2 * M] = np.float32(1e-42)                   # a denormal among normals
    (mask,), obj = run_masks(tm.tmask_exact, [w], N, M)
    _, oobj, opb = oracle.exact(w, N, M, per_block=True, threads=8)
    _check_exact(w, mask, N, M, opb)


@pytest.mark.parametrize("kind", ["f32", "bf16"])
@pytest.mark.parametrize("zeros", [0.5, 0.9, 0.99])
@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (4, 8), (3, 8), (8, 16), (5, 16), (16, 32), (8, 32)])
def test_exact_on_unstructured_sparse_matrices(N, M, zeros, kind):
    """Sec. 5's use: a matrix that is already unstructured-sparse.  Most costs are zero and equal, columns look alike,
    and the cut of many columns falls among the zeros: the optimum must still be reached."""
    w = _inputs(kind, 4 * M, 32 * M, seed=2300 + M + N)
    rng = np.random.default_rng(2301 + M)
    w[rng.random(w.shape) < zeros] = 0
    (mask,), obj = run_masks(tm.tmask_exact, [w], N, M)
    _, oobj, opb = oracle.exact(w, N, M, per_block=True, threads=8)
    _check_exact(w, mask, N, M, opb)
    assert obj[0] == pytest.approx(oobj, rel=1e-5, abs=1e-30)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("N,M", NM)
def test_exact_structured_blocks(N, M, dt):
    """Blocks on which "every column prunes its lightest rows" is as lopsided as it gets (whole rows lighter than
    the others by factors up to 2^-40, products a_i * b_j, one dominant row or column, a checkerboard of two
    values): the start under row prices must stay a valid start whatever it does to them."""
    rng = np.random.default_rng(2500 + M)
    rows, cols = 3 * M, 64 * M
    w = rng.standard_normal((rows, cols)).astype(np.float32)
    i = np.arange(rows)[:, None] % M
    j = np.arange(cols)[None, :] % M
    nb = cols // M
    for b in range(nb):
        c = slice(b * M, (b + 1) * M)
        k = b % 8
        if k == 0:
            w[:, c] *= np.float32(2.0) ** (-(i * (1 + b % 5))).astype(np.float32)     # geometric row scales
        elif k == 1:
            w[:, c] = (1.0 + i) * (1.0 + j[:, c]) * np.float32(0.01)                   # rank one, many equal sums
        elif k == 2:
            w[:, c] *= np.where(i == b % M, np.float32(1e6), np.float32(1.0))          # one dominant row
        elif k == 3:
            w[:, c] *= np.where(j[:, c] == b % M, np.float32(1e6), np.float32(1.0))    # one dominant column
        elif k == 4:
            w[:, c] = np.where((i + j[:, c]) % 2 == 0, np.float32(3.0), np.float32(1.0))
        elif k == 5:
            w[:, c] *= np.float32(2.0) ** (-40.0 * (i >= M // 2)).astype(np.float32)    # half the rows negligible
        elif k == 6:
            w[:, c] = np.round(w[:, c] * 2.0) / 2.0                                     # few distinct values
    if dt == "bf16":
        w = wl.f32_to_bf16_bits(w)
    (mask,), obj = run_masks(tm.tmask_exact, [w], N, M)
    _, oobj, opb = oracle.exact(w, N, M, per_block=True, threads=8)
    _check_exact(w, mask, N, M, opb)
    assert obj[0] == pytest.approx(oobj, rel=1e-5)


@pytest.mark.parametrize("N,M", NM)
def test_exact_is_deterministic(N, M):
    # tie-heavy input has many equally good masks; the same call must return the same one every time (the sort of
    # blocks inside a workgroup and the searches use no atomics and no arrival order)
    w = _inputs("ties_bf16", 6 * M, 2064, seed=2600 + M)
    first = None
    for rep in range(3):
        (mask,), obj = run_masks(tm.tmask_exact, [w], N, M)
        if first is None:
            first = (mask.copy(), obj.copy())
        else:
            assert np.array_equal(mask, first[0]) and np.array_equal(obj, first[1])


def test_exact_non_finite_stays_valid():
    w = wl.special_values_f32(32, 256, seed=2300)
    for N, M in NM:
        (mask,), _ = run_masks(tm.tmask_exact, [w], N, M, with_objective=False)
        b = refs.to_blocks(mask, M)
        assert np.all(b.sum(axis=3) == N) and np.all(b.sum(axis=2) == N)


@pytest.mark.parametrize("kind", ["f32", "bf16"])
def test_exact_batched(kind):
    # several matrices in one launch, rows wider than the matrices; the third one fills more than one workgroup at
    # every N:M (at bf16 8:16 a lane takes half a strip and the launch has twice the workgroups)
    ws = [_inputs(kind, 32, 48, 2400), _inputs(kind, 16, 1040, 2401), _inputs(kind, 64, 1024, 2402)]
    for N, M in NM:
        for fmt in FMTS:
            masks, obj = run_masks(tm.tmask_exact, ws, N, M, fmt, ld_pad=16)
            for k, w in enumerate(ws):
                _, oobj, opb = oracle.exact(w, N, M, per_block=True, threads=8)
                _check_exact(w, masks[k], N, M, opb)
                assert obj[k] == pytest.approx(oobj, rel=1e-5)
            assert obj[k] == pytest.approx(oobj, rel=1e-5)


# ---------------------------------------------------------------- score ------------------------

@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("N,M", NM)
@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_score_matches_oracle(dt, N, M, fmt):
    ws = [_inputs(dt, 5 * M, 1008, seed=3000 + M), _inputs(dt, 2 * M, 64, seed=3001)]
    rng = np.random.default_rng(3002)
    masks = [oracle.approx(ws[0], N, M)[0], (rng.random(ws[1].shape) < 0.55).astype(np.uint8)]
    scores, pbs = run_score(ws, masks, N, M, fmt)
    for w, m, sc, pb in zip(ws, masks, scores, pbs):
        o = oracle.score(w, m, N, M)
        assert sc["retained_l1"] == pytest.approx(o.retained_l1, rel=1e-5)
        assert sc["total_l1"] == pytest.approx(o.total_l1, rel=1e-5)
        assert (sc["kept"], sc["row_violations"], sc["col_violations"], sc["row_not_n"], sc["col_not_n"]) == \
               (o.kept, o.row_violations, o.col_violations, o.row_not_n, o.col_not_n)
        np.testing.assert_allclose(pb, o.per_block, rtol=1e-5, atol=1e-30)


def test_score_bf16_2of4_any_nonzero_byte_is_kept_and_pruned_non_finite_stays_out():
    # mask bytes other than 0 / 1 count as kept; pruned Inf / NaN entries must not reach the retained sum
    N, M = 2, 4
    w = wl.f32_to_bf16_bits(wl.gaussian_f32(5 * M, 1008, seed=3050, std=0.02))
    rng = np.random.default_rng(3051)
    keep = rng.random(w.shape) < 0.5
    bad = rng.random(w.shape) < 0.01
    keep &= ~bad
    w[bad] = rng.choice(np.array([0x7F80, 0xFF80, 0x7FC0, 0x0001], dtype=np.uint16), size=int(bad.sum()))
    mask = np.where(keep, rng.choice(np.array([1, 2, 7, 128, 255], dtype=np.uint8), size=w.shape), 0).astype(np.uint8)
    (sc,), (pb,) = run_score([w], [mask], N, M)
    o = oracle.score(w, (mask != 0).astype(np.uint8), N, M)
    assert (sc["kept"], sc["row_violations"], sc["col_violations"], sc["row_not_n"], sc["col_not_n"]) == \
           (o.kept, o.row_violations, o.col_violations, o.row_not_n, o.col_not_n)
    assert np.isfinite(o.retained_l1) and sc["retained_l1"] == pytest.approx(o.retained_l1, rel=1e-5)
    np.testing.assert_allclose(pb, o.per_block, rtol=1e-5, atol=1e-30)


@pytest.mark.parametrize("dt,rows,cols", [("f32", 4100, 8200), ("bf16", 8196, 8200)])
def test_score_of_a_large_matrix_goes_through_the_two_launch_reduction(dt, rows, cols):
    # more than 8192 workgroup records for one matrix, next to a small one in the same call; random masks, so every
    # counter is non-trivial
    N, M = 2, 4
    ws = [_inputs(dt, rows, cols, seed=3060), _inputs(dt, 8, 64, seed=3061)]
    rng = np.random.default_rng(3062)
    masks = [(rng.random(w.shape) < 0.5).astype(np.uint8) for w in ws]
    scores, pbs = run_score(ws, masks, N, M)
    for w, m, sc, pb in zip(ws, masks, scores, pbs):
        o = oracle.score(w, m, N, M)
        assert sc["retained_l1"] == pytest.approx(o.retained_l1, rel=1e-6)
        assert sc["total_l1"] == pytest.approx(o.total_l1, rel=1e-6)
        assert (sc["kept"], sc["row_violations"], sc["col_violations"], sc["row_not_n"], sc["col_not_n"]) == \
               (o.kept, o.row_violations, o.col_violations, o.row_not_n, o.col_not_n)
        np.testing.assert_allclose(pb, o.per_block, rtol=1e-5, atol=1e-30)


# ---------------------------------------------------------------- error paths (host-side) ------

def test_argument_errors_leave_outputs_untouched():
    w = torch.zeros((16, 32), dtype=torch.float32, device="cuda")
    mask = torch.full((16, 32), 7, dtype=torch.uint8, device="cuda")
    cases = [
        (lambda: tm.tmask_approx([w], [mask], 2, 5), tm.TMASK_ERR_NM),
        (lambda: tm.tmask_approx([w], [mask], 4, 4), tm.TMASK_ERR_NM),
        (lambda: tm.tmask_approx([w[:12]], [mask[:12]], 4, 8), tm.TMASK_ERR_SHAPE),
        (lambda: tm.tmask_approx([w], [mask], 2, 4, objective=torch.zeros(1, dtype=torch.float64, device="cuda")),
         tm.TMASK_ERR_WORKSPACE),
        (lambda: tm.tmask_exact([w], [mask[:, :16].contiguous()], 2, 4), tm.TMASK_ERR_SHAPE),
    ]
    for fn, code in cases:
        with pytest.raises(tm.TmaskError) as e:
            fn()
        assert e.value.code == code, str(e.value)
    torch.cuda.synchronize()
    assert bool((mask == 7).all())
    # a 64 x 147 stem-conv shape is not a multiple of 4 wide: rejected, the caller keeps it dense
    stem = torch.zeros((64, 148), dtype=torch.float32, device="cuda")[:, :147]
    with pytest.raises(tm.TmaskError) as e:
        tm.tmask_approx([stem], [torch.zeros((64, 147), dtype=torch.uint8, device="cuda")], 2, 4)
    assert e.value.code == tm.TMASK_ERR_SHAPE


# ---------------------------------------------------------------- 1-D (non-transposable) pruning

@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("N,M", NM + [(1, 4), (3, 4), (2, 8), (5, 8), (7, 8), (3, 16)])
@pytest.mark.parametrize("kind", ["f32", "bf16", "ties", "ties_bf16", "special"])
def test_prune_1d_bit_exact_ragged(kind, N, M, fmt):
    w = _inputs(kind, 5 * M, 1008, seed=1900 + M)
    (mask,), obj = run_masks(tm.tmask_prune_1d, [w], N, M, fmt)
    omask, oobj = oracle.prune_1d(w, N, M)
    assert np.array_equal(mask, omask)
    if kind != "special":
        assert obj[0] == pytest.approx(oobj, rel=1e-5)


def test_prune_1d_batched_with_strides():
    rng = np.random.default_rng(19)
    shapes = [(16, 16), (16, 32), (64, 48), (144, 272), (32, 1040)]
    ws = [_inputs("bf16" if k % 2 else "f32", *shapes[int(rng.integers(len(shapes)))], seed=1950 + k) for k in range(6)]
    for group in (ws[0::2], ws[1::2]):                      # one dtype per call
        masks, obj = run_masks(tm.tmask_prune_1d, group, 4, 8, ld_pad=32)
        for w, m, o in zip(group, masks, obj):
            omask, oobj = oracle.prune_1d(w, 4, 8)
            assert np.array_equal(m, omask)
            assert o == pytest.approx(oobj, rel=1e-5)

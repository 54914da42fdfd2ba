"""Seeded random draws of (data kind, N:M, shape, padding of the leading dimension, mask format) through the mask
entry points and the score, each against the oracle: the combinations that the hand-picked cases leave out (every N
at every M, tie-heavy data at general N, bit masks with padded rows)."""
import numpy as np
import pytest

import oracle
from paper_2102_08124_amd import workloads as wl
from tests import refs

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2102_08124_amd import binding as tm   # noqa: E402
from tests.gpu_util import run_masks, run_score  # noqa: E402

KINDS = ("f32", "bf16", "ties", "ties_bf16", "sparse", "sparse_bf16")


def _draw(kind, rows, cols, seed):
    if kind == "f32":
        return wl.gaussian_f32(rows, cols, seed)
    if kind == "bf16":
        return wl.f32_to_bf16_bits(wl.gaussian_f32(rows, cols, seed, std=0.02))
    if kind == "ties":
        return wl.tie_heavy_f32(rows, cols, seed, levels=4)
    if kind == "ties_bf16":
        return wl.f32_to_bf16_bits(wl.tie_heavy_f32(rows, cols, seed, levels=3))
    w = wl.gaussian_f32(rows, cols, seed)                    # unstructured-sparse: 80 % exact zeros
    w[np.random.default_rng(seed + 1).random(w.shape) < 0.8] = 0.0
    return w if kind == "sparse" else wl.f32_to_bf16_bits(w)


def _cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for k in range(n):
        M = int(rng.choice([4, 8, 16, 32]))
        N = int(rng.integers(1, M))
        kind = KINDS[int(rng.integers(len(KINDS)))]
        per16 = 4 if "bf16" not in kind else 8             # columns in 16 bytes: keeps the strip kernels eligible
        step = int(np.lcm(M, 8))                           # whole bytes per row of a bit mask
        rows = M * int(rng.integers(1, 5))
        cols = step * int(rng.integers(1, 1 + 640 // step))
        pad = int(rng.choice([0, 0, per16 * 4, per16 * 12]))
        fmt = int(rng.choice([tm.TMASK_MASK_U8, tm.TMASK_MASK_BITS]))
        out.append(pytest.param(kind, N, M, rows, cols, pad, fmt, 9000 + k, id="%s-%d:%d-%dx%d-pad%d-fmt%d" % (kind, N, M, rows, cols, pad, fmt)))
    return out


@pytest.mark.parametrize("kind,N,M,rows,cols,pad,fmt,seed", _cases(96, 424242))
def test_random_configuration(kind, N, M, rows, cols, pad, fmt, seed):
    w = _draw(kind, rows, cols, seed)
    # Algorithm 1: bit-exact
    (amask,), aobj = run_masks(tm.tmask_approx, [w], N, M, fmt, ld_pad=pad)
    omask, oobj = oracle.approx(w, N, M)
    assert np.array_equal(amask, omask)
    assert aobj[0] == pytest.approx(oobj, rel=1e-5, abs=1e-30)
    # row pruning: bit-exact
    (pmask,), pobj = run_masks(tm.tmask_prune_1d, [w], N, M, fmt, ld_pad=pad)
    opmask, opobj = oracle.prune_1d(w, N, M)[:2]
    assert np.array_equal(pmask, opmask)
    assert pobj[0] == pytest.approx(opobj, rel=1e-5, abs=1e-30)
    # exact: valid, and every block's retained L1 is the optimum
    (emask,), eobj = run_masks(tm.tmask_exact, [w], N, M, fmt, ld_pad=pad)
    _, oeobj, opb = oracle.exact(w, N, M, per_block=True, threads=8)
    b = refs.to_blocks(emask, M)
    assert np.all(b.sum(axis=3) == N) and np.all(b.sum(axis=2) == N)
    np.testing.assert_allclose(refs.per_block_sums(refs.magnitudes(w) * emask, M), opb, rtol=1e-5, atol=1e-30)
    assert eobj[0] == pytest.approx(oeobj, rel=1e-5, abs=1e-30)
    # score of Algorithm 1's mask
    (sc,), (pb,) = run_score([w], [amask], N, M, fmt)
    o = oracle.score(w, amask, N, M)
    assert (sc["kept"], sc["row_violations"], sc["col_violations"], sc["row_not_n"], sc["col_not_n"]) == \
           (o.kept, o.row_violations, o.col_violations, o.row_not_n, o.col_not_n)
    assert sc["retained_l1"] == pytest.approx(o.retained_l1, rel=1e-5, abs=1e-30)
    np.testing.assert_allclose(pb, o.per_block, rtol=1e-5, atol=1e-30)

"""GPU parity for tmask_apply_pack: every output byte equals the oracle's."""
import numpy as np
import pytest

import oracle
from paper_2102_08124_amd import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2102_08124_amd import binding as tm   # noqa: E402
from tests.gpu_util import run_pack              # noqa: E402


def _w(dt, rows, cols, seed):
    w = wl.gaussian_f32(rows, cols, seed, std=0.02)
    w[0, 0] = -0.0
    return w if dt == "f32" else wl.f32_to_bf16_bits(w)


def _same(got, want):
    for g, o, name in zip(got, want, ("vals", "idx", "valsT", "idxT")):
        assert g.shape == o.shape, name
        assert np.array_equal(g.view(np.uint8), o.view(np.uint8)), name


@pytest.mark.parametrize("fmt", [tm.TMASK_MASK_U8, tm.TMASK_MASK_BITS])
@pytest.mark.parametrize("N,M", [(2, 4), (4, 8), (8, 16)])
@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_pack_matches_oracle_ragged(dt, N, M, fmt):
    # 5 block-rows x 1008 columns: partial tiles on both edges
    w = _w(dt, 5 * M, 1008, seed=4000 + M)
    for mask in (oracle.approx(w, N, M)[0], oracle.exact(w, N, M, threads=8)[0]):
        (got,) = run_pack([w], [mask], N, M, fmt)
        _same(got, oracle.apply_pack(w, mask, N, M))


@pytest.mark.parametrize("N,M", [(1, 4), (3, 4), (3, 8), (7, 8), (1, 16), (5, 16), (15, 16)])
def test_pack_other_n(N, M):
    for dt in ("f32", "bf16"):
        w = _w(dt, 8 * M + M, 272, seed=4100 + N)      # cols/M*N odd in places: element-wise store path
        mask = oracle.approx(w, N, M)[0]
        (got,) = run_pack([w], [mask], N, M)
        _same(got, oracle.apply_pack(w, mask, N, M))


def test_pack_non_finite_and_empty_mask():
    w = wl.special_values_f32(64, 128, seed=4200)
    mask = oracle.approx(w, 2, 4)[0]
    (got,) = run_pack([w], [mask], 2, 4)
    _same(got, oracle.apply_pack(w, mask, 2, 4))       # pruned NaN/Inf become +0
    zero = np.zeros_like(mask)
    (got,) = run_pack([w], [zero], 2, 4)
    _same(got, oracle.apply_pack(w, zero, 2, 4))
    full = np.ones_like(mask)                          # more than N kept: the first N of each group win
    (got,) = run_pack([w], [full], 2, 4)
    _same(got, oracle.apply_pack(w, full, 2, 4))


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_pack_batched_with_strides(dt):
    rng = np.random.default_rng(9)
    shapes = [(16, 16), (16, 32), (64, 48), (144, 272), (32, 1040), (256, 64)]
    ws = [_w(dt, *shapes[int(rng.integers(len(shapes)))], seed=4300 + k) for k in range(40)]   # > one 32-matrix launch
    for N, M in ((2, 4), (4, 8), (8, 16)):
        masks = [oracle.approx(w, N, M)[0] for w in ws]
        got = run_pack(ws, masks, N, M, ld_pad=32)
        for k, w in enumerate(ws):
            _same(got[k], oracle.apply_pack(w, masks[k], N, M))


def test_pack_roundtrip_and_l1():
    w = wl.gaussian_f32(128, 256, seed=4400)
    mask, obj = oracle.exact(w, 4, 8, threads=4)
    (got,) = run_pack([w], [mask], 4, 8)
    vals, idx, valsT, idxT = got
    masked = np.where(mask != 0, w, np.float32(0))
    assert np.array_equal(oracle.unpack(vals, idx, 128, 256, 4, 8), masked)
    assert np.array_equal(oracle.unpack(valsT, idxT, 256, 128, 4, 8), masked.T)
    assert np.abs(vals.astype(np.float64)).sum() == pytest.approx(obj, rel=1e-12)


@pytest.mark.parametrize("fmt", [tm.TMASK_MASK_U8, tm.TMASK_MASK_BITS])
@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_pack48_multi_tile_and_degenerate_masks(dt, fmt):
    # several whole tiles of the 4:8 kernels (bf16: 128 rows x 256 columns, fp32: 64 x 256) plus ragged edges in
    # both directions; masks with 0 to 8 kept entries per group exercise fillers and the "first four win" rule
    w = wl.special_values_f32(392, 776, seed=4500)
    if dt == "bf16":
        w = wl.f32_to_bf16_bits(w)
    rng = np.random.default_rng(45)
    masks = [oracle.approx(w, 4, 8)[0],
             (rng.random(w.shape) < 0.5).astype(np.uint8),      # unstructured: 0 to 8 kept per group
             np.zeros(w.shape, dtype=np.uint8), np.ones(w.shape, dtype=np.uint8)]
    masks[1][:, :16] = 0
    masks[1][:16, :] = 1
    for mask in masks:
        (got,) = run_pack([w], [mask], 4, 8, fmt)
        _same(got, oracle.apply_pack(w, mask, 4, 8))


@pytest.mark.parametrize("dt,N,M", [("f32", 2, 4), ("bf16", 2, 4), ("bf16", 4, 8), ("f32", 4, 8)])
def test_pack_tile_order_bands_and_runs(dt, N, M):
    # 4352 x 2304: nine tile columns (one group of eight bands plus a ninth band) and more tile rows than one
    # vertical run of 4096 rows, so every branch of the tile numbering is taken; the fused call shares it
    w = _w(dt, 4352, 2304, seed=4600 + M)
    mask = oracle.approx(w, N, M)[0]
    want = oracle.apply_pack(w, mask, N, M)
    (got,) = run_pack([w], [mask], N, M)
    _same(got, want)
    from tests.gpu_util import run_fused
    got_f, _, _ = run_fused([w], N, M, with_mask=(M != 4), with_objective=False)
    _same(got_f[0], want)


@pytest.mark.parametrize("dt,N,M", [("f32", 2, 4), ("bf16", 2, 4), ("bf16", 4, 8), ("f32", 4, 8)])
def test_pack_and_one_pass_random_shapes(dt, N, M):
    # a batch of matrices with random (seeded) shapes, from a single block to several tiles either way, with row
    # strides wider than the rows; apply_pack with unstructured masks, the one-pass call against the oracle's pair
    rng = np.random.default_rng(4700 + M)
    step = 8 if dt == "bf16" else 4                    # 16-byte rows
    step = max(step, M)
    shapes = [(int(rng.integers(1, 40)) * M, int(rng.integers(1, 150)) * step) for _ in range(10)]
    shapes += [(M, step), (M * 33, step), (M, step * 130)]
    ws = [_w(dt, r, c, seed=4710 + k) for k, (r, c) in enumerate(shapes)]
    masks = [(rng.random(w.shape) < 0.5).astype(np.uint8) for w in ws]
    got = run_pack(ws, masks, N, M, ld_pad=40)
    for k, w in enumerate(ws):
        _same(got[k], oracle.apply_pack(w, masks[k], N, M))
    from tests.gpu_util import run_fused
    got_f, gmasks, _ = run_fused(ws, N, M, ld_pad=40)
    for k, w in enumerate(ws):
        om = oracle.approx(w, N, M)[0]
        assert np.array_equal(gmasks[k] != 0, om != 0), k
        _same(got_f[k], oracle.apply_pack(w, om, N, M))


@pytest.mark.parametrize("N,M", [(2, 4), (4, 8), (8, 16)])
@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_pack_outputs_only_four_byte_aligned(dt, N, M):
    # vals and valsT four bytes off a 16-byte boundary: the specialised kernels (8-byte stores) and the 16-byte
    # stores of the general one must step aside for the element-wise path; same bytes as ever
    from tests.gpu_util import to_dev, mask_to_dev
    w = _w(dt, 6 * M, 272, seed=4800 + M)
    mask = oracle.approx(w, N, M)[0]
    wd = to_dev(w)
    vs, is_, vts, its = tm.packed_shapes(w.shape[0], w.shape[1], N, M)
    off = 1 if dt == "f32" else 2                      # elements = four bytes
    def shifted(shape):
        n = int(np.prod(shape))
        buf = torch.zeros(n + 8, dtype=wd.dtype, device="cuda")
        return buf[off:off + n].view(*shape)
    packed = (shifted(vs), torch.zeros(is_, dtype=torch.uint8, device="cuda"),
              shifted(vts), torch.zeros(its, dtype=torch.uint8, device="cuda"))
    assert packed[0].data_ptr() % 16 == 4 and packed[2].data_ptr() % 16 == 4
    tm.tmask_apply_pack([wd], [mask_to_dev(mask, tm.TMASK_MASK_U8)], [packed], N, M)
    torch.cuda.synchronize()
    got = []
    for t in packed:
        got.append(t.view(torch.int16).cpu().numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.cpu().numpy())
    _same(tuple(got), oracle.apply_pack(w, mask, N, M))

"""GPU parity for tmask_approx_pack: Algorithm 1 and the compression in one call give exactly what the
oracle's Algorithm 1 followed by the oracle's compression gives (every byte), plus the mask and objective."""
import ctypes

import numpy as np
import pytest

import oracle
from paper_2102_08124_amd import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2102_08124_amd import binding as tm        # noqa: E402
from tests.gpu_util import run_fused, to_dev          # noqa: E402


def _w(dt, rows, cols, seed):
    w = wl.gaussian_f32(rows, cols, seed, std=0.02)
    w[0, 0] = -0.0
    return w if dt == "f32" else wl.f32_to_bf16_bits(w)


def _check(ws, N, M, got, masks, objs, with_mask=True):
    for k, w in enumerate(ws):
        omask, oobj = oracle.approx(w, N, M)
        want = oracle.apply_pack(w, omask, N, M)
        for g, o, name in zip(got[k], want, ("vals", "idx", "valsT", "idxT")):
            assert g.shape == o.shape, (k, name)
            assert np.array_equal(g.view(np.uint8), o.view(np.uint8)), (k, name)
        if with_mask:
            assert np.array_equal(masks[k] != 0, omask != 0), k
        if objs is not None:
            if np.isnan(oobj):
                assert np.isnan(objs[k])
            else:
                assert objs[k] == pytest.approx(oobj, rel=1e-5, abs=1e-30), k


@pytest.mark.parametrize("with_mask", [True, False])
@pytest.mark.parametrize("fmt", [tm.TMASK_MASK_U8, tm.TMASK_MASK_BITS])
@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_fused_2of4_ragged(dt, fmt, with_mask):
    # 68 x 1032: one full tile row plus one block-row, partial tiles on the right edge for both dtypes;
    # 192 x 1024: interior tiles only (the copy of the loop without bounds tests)
    ws = [_w(dt, 68, 1032, seed=5000), _w(dt, 192, 1024, seed=5001), _w(dt, 4, 8, seed=5002)]
    got, masks, objs = run_fused(ws, 2, 4, fmt, with_mask=with_mask)
    _check(ws, 2, 4, got, masks, objs, with_mask)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_fused_2of4_ties_and_special_values(dt):
    ties = wl.tie_heavy_f32(128, 528, seed=5100)
    spec = wl.special_values_f32(64, 264, seed=5101)
    zeros = np.zeros((64, 256), dtype=np.float32)
    ws = [ties, spec, zeros]
    if dt == "bf16":
        ws = [wl.f32_to_bf16_bits(w) for w in ws]
    got, masks, objs = run_fused(ws, 2, 4)
    _check(ws, 2, 4, got, masks, objs)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_fused_batched_with_strides_and_no_objective(dt):
    rng = np.random.default_rng(11)
    shapes = [(16, 16), (16, 32), (64, 48), (144, 272), (32, 1040), (256, 64), (64, 512)]
    ws = [_w(dt, *shapes[int(rng.integers(len(shapes)))], seed=5200 + k) for k in range(70)]   # more than one launch
    got, masks, objs = run_fused(ws, 2, 4, ld_pad=32)
    _check(ws, 2, 4, got, masks, objs)
    got, masks, objs = run_fused(ws[:5], 2, 4, with_mask=False, with_objective=False)
    _check(ws[:5], 2, 4, got, masks, objs, with_mask=False)


@pytest.mark.parametrize("with_mask", [True, False])
@pytest.mark.parametrize("fmt", [tm.TMASK_MASK_U8, tm.TMASK_MASK_BITS])
@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_fused_4of8_one_pass(dt, fmt, with_mask):
    # 4:8 has one-pass kernels of its own (bf16: 128 x 256 tiles, fp32: 64 x 256): whole tiles, ragged edges, a
    # single block, and tie-heavy matrices with special values (the index tie-break decides many entries there;
    # at fp32 a tie across a cut sends the whole wavefront through the rank form)
    conv = (lambda w: wl.f32_to_bf16_bits(w)) if dt == "bf16" else (lambda w: w)
    ws = [_w(dt, 392, 776, seed=5200), _w(dt, 256, 512, seed=5201), _w(dt, 8, 8, seed=5202),
          conv(wl.tie_heavy_f32(136, 264, seed=5203)), conv(wl.special_values_f32(64, 128, seed=5204))]
    got, masks, objs = run_fused(ws, 4, 8, fmt, with_mask=with_mask, ld_pad=24)
    _check(ws, 4, 8, got, masks, objs, with_mask)


@pytest.mark.parametrize("dt,N,M", [("f32", 2, 4), ("bf16", 2, 4), ("f32", 4, 8), ("bf16", 4, 8)])
def test_fused_tall_narrow_with_objective(dt, N, M):
    # one block column, thousands of block rows: the one-pass kernels keep one partial sum per tile of 64 or 128
    # rows, many more than the mask kernels' tiles of 256 strips; a workspace sized by tmask_workspace_bytes holds them
    ws = [_w(dt, 16384, 8, seed=5250 + M)]
    got, masks, objs = run_fused(ws, N, M)
    _check(ws, N, M, got, masks, objs)


@pytest.mark.parametrize("N,M", [(8, 16), (1, 4), (3, 4), (5, 8)])
def test_fused_other_nm_runs_both_steps(N, M):
    for dt in ("f32", "bf16"):
        ws = [_w(dt, 5 * M, 272, seed=5300 + N), _w(dt, 8 * M, 1008, seed=5301 + N)]
        got, masks, objs = run_fused(ws, N, M)
        _check(ws, N, M, got, masks, objs)


def test_fused_config1_matches_separate_calls():
    w = wl.config1()
    got, masks, objs = run_fused([w], 2, 4)
    _check([w], 2, 4, got, masks, objs)
    # the same through the two separate entry points
    wd = to_dev(w)
    m = tm.alloc_masks([wd])[0]
    tm.tmask_approx([wd], [m], 2, 4)
    pk = tm.alloc_packed(wd, 2, 4)
    tm.tmask_apply_pack([wd], [m], [pk], 2, 4)
    torch.cuda.synchronize()
    for a, b in zip(got[0], pk):
        assert np.array_equal(a.view(np.uint8), b.cpu().numpy().view(np.uint8))


def test_fused_argument_errors():
    w = to_dev(_w("f32", 16, 16, seed=5400))
    w2 = to_dev(_w("f32", 16, 16, seed=5401))
    pk, pk2 = tm.alloc_packed(w, 2, 4), tm.alloc_packed(w2, 2, 4)
    m = tm.alloc_masks([w])[0]
    lib = tm.load_library()
    # mask for one matrix only
    arr = (tm.tmask_fused_desc * 2)()
    arr[0] = tm.tmask_fused_desc(w.data_ptr(), 16, 16, 16, m.data_ptr(), 16, *[t.data_ptr() for t in pk], None)
    arr[1] = tm.tmask_fused_desc(w2.data_ptr(), 16, 16, 16, None, 0, *[t.data_ptr() for t in pk2], None)
    assert lib.tmask_approx_pack(arr, 2, tm.TMASK_F32, 2, 4, tm.TMASK_MASK_U8, None, 0, None) == tm.TMASK_ERR_NULL
    # other N:M without mask buffers
    w8 = to_dev(_w("f32", 16, 16, seed=5402))
    with pytest.raises(tm.TmaskError) as e:
        tm.tmask_approx_pack([w8], None, [tm.alloc_packed(w8, 8, 16)], 8, 16)
    assert e.value.code == tm.TMASK_ERR_NULL
    # objective without workspace
    obj = torch.zeros(1, dtype=torch.float64, device="cuda")
    with pytest.raises(tm.TmaskError) as e:
        tm.tmask_approx_pack([w], None, [pk], 2, 4, objective=obj)
    assert e.value.code == tm.TMASK_ERR_WORKSPACE
    # vals not 8-byte aligned: the one-pass kernel cannot write it, the two-step path needs the mask buffers
    vals_off = torch.empty(16 * 8 + 1, dtype=torch.float32, device="cuda")[1:].view(16, 8)
    arr1 = (tm.tmask_fused_desc * 1)()
    arr1[0] = tm.tmask_fused_desc(w.data_ptr(), 16, 16, 16, None, 0, vals_off.data_ptr(), pk[1].data_ptr(),
                                  pk[2].data_ptr(), pk[3].data_ptr(), None)
    assert lib.tmask_approx_pack(arr1, 1, tm.TMASK_F32, 2, 4, tm.TMASK_MASK_U8, None, 0, None) == tm.TMASK_ERR_NULL
    # a NULL packed output
    arr1[0] = tm.tmask_fused_desc(w.data_ptr(), 16, 16, 16, None, 0, None, pk[1].data_ptr(), pk[2].data_ptr(),
                                  pk[3].data_ptr(), None)
    assert lib.tmask_approx_pack(arr1, 1, tm.TMASK_F32, 2, 4, tm.TMASK_MASK_U8, None, 0, None) == tm.TMASK_ERR_NULL
    torch.cuda.synchronize()
    # nothing was written by the rejected calls
    assert ctypes.sizeof(tm.tmask_fused_desc) == 88

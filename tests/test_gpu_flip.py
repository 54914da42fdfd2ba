"""GPU parity for tmask_flip_count: exact counts against the oracle's definition."""
import numpy as np
import pytest

import oracle
from paper_2102_08124_amd import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2102_08124_amd import binding as tm            # noqa: E402
from tests.gpu_util import mask_to_dev                     # noqa: E402


def _masks(rows, cols, seed, p_flip=0.1):
    rng = np.random.default_rng(seed)
    a = (rng.random((rows, cols)) < 0.5).astype(np.uint8)
    b = np.where(rng.random((rows, cols)) < p_flip, 1 - a, a).astype(np.uint8)
    a[a != 0] = rng.integers(1, 256, size=int((a != 0).sum()), dtype=np.uint8)     # any non-zero byte counts as kept
    return a, b


@pytest.mark.parametrize("fmt", [tm.TMASK_MASK_U8, tm.TMASK_MASK_BITS])
def test_flip_count_batch_of_shapes(fmt):
    shapes = [(64, 64), (5, 1008), (128, 4096), (3, 8), (17, 24), (1024, 1040)]
    pairs = [_masks(r, c, seed=7000 + k) for k, (r, c) in enumerate(shapes)]
    pairs.append((pairs[0][0], pairs[0][0]))                       # identical masks: zero flips
    flips = torch.full((len(pairs),), -5, dtype=torch.int64, device="cuda")
    if fmt == tm.TMASK_MASK_BITS:
        da = [mask_to_dev((a != 0).astype(np.uint8), fmt) for a, _ in pairs]
        db = [mask_to_dev((b != 0).astype(np.uint8), fmt) for _, b in pairs]
    else:
        da = [torch.from_numpy(a).cuda() for a, _ in pairs]
        db = [torch.from_numpy(b).cuda() for _, b in pairs]
    tm.tmask_flip_count(da, db, [a.shape[1] for a, _ in pairs], flips, mask_fmt=fmt)
    torch.cuda.synchronize()
    got = flips.cpu().numpy()
    for k, (a, b) in enumerate(pairs):
        assert int(got[k]) == oracle.flip_count(a, b), k


def test_flip_count_strided_views_and_config5_step():
    # masks that are column slices of wider buffers (row stride > cols, 4-byte aligned only)
    a, b = _masks(96, 260, seed=7100)
    bufa = torch.zeros((96, 300), dtype=torch.uint8, device="cuda")
    bufb = torch.ones((96, 332), dtype=torch.uint8, device="cuda")
    bufa[:, 4:264] = torch.from_numpy(a).cuda()
    bufb[:, 8:268] = torch.from_numpy(b).cuda()
    flips = torch.zeros(1, dtype=torch.int64, device="cuda")
    tm.tmask_flip_count([bufa[:, 4:264]], [bufb[:, 8:268]], [260], flips)
    torch.cuda.synchronize()
    assert int(flips[0]) == oracle.flip_count(a, b)
    # two consecutive masks of the drifting-weights workload, computed on the device
    w0 = wl.f32_to_bf16_bits(wl.gaussian_f32(256, 512, seed=7200, std=0.02))
    w1 = wl.f32_to_bf16_bits(wl.gaussian_f32(256, 512, seed=7200, std=0.02) +
                             1e-3 * wl.gaussian_f32(256, 512, seed=7201, std=0.02))
    from tests.gpu_util import to_dev
    d0, d1 = to_dev(w0), to_dev(w1)
    m0, m1 = tm.alloc_masks([d0])[0], tm.alloc_masks([d1])[0]
    tm.tmask_approx([d0], [m0], 2, 4)
    tm.tmask_approx([d1], [m1], 2, 4)
    tm.tmask_flip_count([m0], [m1], [512], flips)
    torch.cuda.synchronize()
    assert int(flips[0]) == oracle.flip_count(oracle.approx(w0, 2, 4)[0], oracle.approx(w1, 2, 4)[0])


def test_flip_count_argument_errors():
    a = torch.zeros((8, 16), dtype=torch.uint8, device="cuda")
    flips = torch.zeros(1, dtype=torch.int64, device="cuda")
    lib = tm.load_library()
    arr = (tm.tmask_flip_desc * 1)()
    arr[0] = tm.tmask_flip_desc(a.data_ptr(), 16, None, 16, 8, 16, flips.data_ptr())
    assert lib.tmask_flip_count(arr, 1, tm.TMASK_MASK_U8, None) == tm.TMASK_ERR_NULL
    arr[0] = tm.tmask_flip_desc(a.data_ptr(), 8, a.data_ptr(), 16, 8, 16, flips.data_ptr())
    assert lib.tmask_flip_count(arr, 1, tm.TMASK_MASK_U8, None) == tm.TMASK_ERR_SHAPE
    arr[0] = tm.tmask_flip_desc(a.data_ptr(), 16, a.data_ptr(), 16, 8, 12, flips.data_ptr())
    assert lib.tmask_flip_count(arr, 1, tm.TMASK_MASK_BITS, None) == tm.TMASK_ERR_SHAPE
    arr[0] = tm.tmask_flip_desc(a.data_ptr(), 16, a.data_ptr(), 16, 8, 16, flips.data_ptr() + 4)
    assert lib.tmask_flip_count(arr, 1, tm.TMASK_MASK_U8, None) == tm.TMASK_ERR_ALIGN
    torch.cuda.synchronize()


def test_dynamic_masks_loop_runs_and_reports(capsys):
    # the drifting-weights loop of the package at a small size: masks per step, flip counts, rates
    import sys
    from paper_2102_08124_amd import dynamic_masks
    argv = sys.argv
    sys.argv = ["dynamic_masks", "--side", "512", "--steps", "4"]
    try:
        dynamic_masks.main()
    finally:
        sys.argv = argv
    out = capsys.readouterr().out
    assert "flip fraction per step" in out and "weights/s" in out

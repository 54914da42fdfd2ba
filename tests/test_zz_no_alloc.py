"""tmask_approx_noalloc (the entry point whose scratch memory is a static device array inside the library) against
tmask_approx (caller workspace): same masks bit for bit, same objectives bit for bit (same kernels, same summation
order), on two calls in a row, the second one smaller, so that what the first call left in the shared array is seen
not to leak into the second.  Runs alone in a fresh process and after the other tests."""
import ctypes

import numpy as np
import pytest

from paper_2102_08124_amd import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2102_08124_amd import binding as tm            # noqa: E402
from tests.gpu_util import to_dev                          # noqa: E402


def _both(ws_np, N, M, fmt):
    ws = [to_dev(w) for w in ws_np]
    n = len(ws)
    ref_masks, got_masks = tm.alloc_masks(ws, fmt), tm.alloc_masks(ws, fmt)
    for m in ref_masks + got_masks:
        m.fill_(0xCD)
    ref_obj = torch.full((n,), -1.0, dtype=torch.float64, device="cuda")
    got_obj = torch.full((n,), -2.0, dtype=torch.float64, device="cuda")
    wsp = tm.alloc_workspace(ws, N, M)
    tm.tmask_approx(ws, ref_masks, N, M, objective=ref_obj, mask_fmt=fmt, workspace=wsp)
    # straight through the C symbol: descriptors, no workspace argument
    batch = tm.MatBatch(ws, got_masks, got_obj)
    rc = tm.load_library().tmask_approx_noalloc(batch.arr, batch.n, batch.dt, N, M, fmt,
                                                ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == tm.TMASK_OK, tm.load_library().tmask_last_error()
    torch.cuda.synchronize()
    for k in range(n):
        assert torch.equal(ref_masks[k], got_masks[k]), "mask %d differs" % k
    ro, go = ref_obj.cpu().numpy(), got_obj.cpu().numpy()
    assert np.array_equal(ro.view(np.uint64), go.view(np.uint64)), (ro, go)     # bit-identical objectives
    assert (ro > 0).all()
    return ro


@pytest.mark.parametrize("fmt", [tm.TMASK_MASK_U8, tm.TMASK_MASK_BITS])
def test_noalloc_matches_workspace_entry_point_two_calls_in_a_row(fmt):
    # first call: a batch of five matrices (fp32 2:4), several workgroups each and ragged tails
    first = [wl.gaussian_f32(r, c, seed=9100 + k) for k, (r, c) in
             enumerate([(256, 1024), (64, 72), (520, 136), (4, 8), (1024, 2048)])]
    o1 = _both(first, 2, 4, fmt)
    # second call, smaller: two matrices; stale partial sums of the first call sit in the array beyond and under them
    second = [wl.gaussian_f32(r, c, seed=9200 + k) for k, (r, c) in enumerate([(128, 264), (8, 16)])]
    o2 = _both(second, 2, 4, fmt)
    assert o2.sum() < o1.sum()
    # and bf16 4:8 after that (another kernel family through the same array)
    third = [wl.f32_to_bf16_bits(wl.gaussian_f32(r, c, seed=9300 + k, std=0.02)) for k, (r, c) in
             enumerate([(512, 512), (64, 136)])]
    _both(third, 4, 8, fmt)
    # M = 32 runs on the column-per-lane kernels: one partial sum per tile of 32 rows x 64 columns
    fourth = [wl.gaussian_f32(r, c, seed=9350 + k) for k, (r, c) in enumerate([(128, 416), (32, 32)])]
    _both(fourth, 16, 32, fmt)


def test_noalloc_rejects_what_does_not_fit_and_needs_no_scratch_without_objective():
    lib = tm.load_library()
    # 65537 workgroups of 256 strips: one more than the array holds -> refused on the host, nothing launched
    # (the descriptor only has to look valid: the check happens before anything is enqueued)
    w = torch.zeros((4, 8), dtype=torch.float32, device="cuda")
    m = torch.zeros((4, 8), dtype=torch.uint8, device="cuda")
    obj = torch.zeros(1, dtype=torch.float64, device="cuda")
    rows = 4 * 65537
    arr = (tm.tmask_mat * 1)()
    arr[0] = tm.tmask_mat(w.data_ptr(), rows, 1024, 1024, m.data_ptr(), 1024, obj.data_ptr())
    rc = lib.tmask_approx_noalloc(arr, 1, tm.TMASK_F32, 2, 4, tm.TMASK_MASK_U8, None)
    assert rc == tm.TMASK_ERR_WORKSPACE
    assert b"65536" in lib.tmask_last_error()
    torch.cuda.synchronize()
    assert float(obj[0]) == 0.0
    # without objectives the array is not used: masks only, equal to tmask_approx's
    w_np = wl.gaussian_f32(64, 128, seed=9400)
    wd = to_dev(w_np)
    a, b = tm.alloc_masks([wd])[0], tm.alloc_masks([wd])[0]
    tm.tmask_approx([wd], [a], 2, 4)
    tm.tmask_approx_noalloc([wd], [b], 2, 4)
    torch.cuda.synchronize()
    assert torch.equal(a, b)

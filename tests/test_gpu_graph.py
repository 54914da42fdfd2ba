"""The four calls of a benchmark step recorded into a HIP graph: every replay must reproduce the eager results."""
import numpy as np
import pytest

from paper_2102_08124_amd import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2102_08124_amd import binding as tm   # noqa: E402


def _state(ws, N, M):
    n = len(ws)
    return {
        "amask": tm.alloc_masks(ws), "emask": tm.alloc_masks(ws),
        "aobj": torch.zeros(n, dtype=torch.float64, device="cuda"),
        "eobj": torch.zeros(n, dtype=torch.float64, device="cuda"),
        "packed": [tm.alloc_packed(w, N, M) for w in ws],
        "sout": torch.zeros(n * tm.SCORE_OUT_BYTES, dtype=torch.uint8, device="cuda"),
    }


def _step(ws, st, wsp, N, M, stream=None):
    tm.tmask_approx(ws, st["amask"], N, M, objective=st["aobj"], workspace=wsp, stream=stream)
    tm.tmask_exact(ws, st["emask"], N, M, objective=st["eobj"], workspace=wsp, stream=stream)
    tm.tmask_apply_pack(ws, st["emask"], st["packed"], N, M, stream=stream)
    tm.tmask_score(ws, st["amask"], N, M, st["sout"], workspace=wsp, stream=stream)


def _snapshot(st):
    out = [m.clone() for m in st["amask"]] + [m.clone() for m in st["emask"]] + [st["aobj"].clone(), st["eobj"].clone(),
                                                                              st["sout"].clone()]
    for pk in st["packed"]:
        out += [t.clone() for t in pk]
    return out


def test_step_in_a_graph_replays_exactly():
    N, M = 2, 4
    shapes = [(64, 64), (128, 576), (256, 1024), (512, 2304)]
    ws = [torch.from_numpy(wl.gaussian_f32(r, c, seed=8000 + k, std=0.05)).cuda() for k, (r, c) in enumerate(shapes)]
    wsp = tm.alloc_workspace(ws, N, M)
    eager = _state(ws, N, M)
    _step(ws, eager, wsp, N, M)
    torch.cuda.synchronize()
    want = _snapshot(eager)

    st = _state(ws, N, M)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        _step(ws, st, wsp, N, M)                  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        _step(ws, st, wsp, N, M)
    for rep in range(4):
        # spoil the outputs and do unrelated eager work between replays
        for m in st["amask"] + st["emask"]:
            m.fill_(0x5A)
        st["aobj"].fill_(-1.0)
        for pk in st["packed"]:
            for t in pk:
                t.view(torch.uint8).fill_(0xEE)
        junk = torch.randn(1 << 20, device="cuda").sum()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = _snapshot(st)
        assert len(got) == len(want)
        for a, b in zip(got, want):
            assert np.array_equal(a.cpu().numpy().view(np.uint8), b.cpu().numpy().view(np.uint8)), rep
        del junk


def test_four_of_eight_calls_in_a_graph_replay_exactly():
    """The 4:8 calls (threshold-network approximation, augmenting paths from a priced start, the 4:8 pack kernel, the
    one-pass compression and the one-pass masked copy) recorded into one graph: replays reproduce the eager run."""
    N, M = 4, 8
    shapes = [(64, 64), (128, 576), (512, 1024)]
    ws = [torch.from_numpy(wl.gaussian_f32(r, c, seed=8100 + k, std=0.05)).cuda() for k, (r, c) in enumerate(shapes)]
    wsp = tm.alloc_workspace(ws, N, M)

    def state():
        n = len(ws)
        return {"amask": tm.alloc_masks(ws), "emask": tm.alloc_masks(ws),
                "aobj": torch.zeros(n, dtype=torch.float64, device="cuda"),
                "eobj": torch.zeros(n, dtype=torch.float64, device="cuda"),
                "packed": [tm.alloc_packed(w, N, M) for w in ws], "fpacked": [tm.alloc_packed(w, N, M) for w in ws],
                "dense": [torch.empty_like(w) for w in ws]}

    def step(st, stream=None):
        tm.tmask_approx(ws, st["amask"], N, M, objective=st["aobj"], workspace=wsp, stream=stream)
        tm.tmask_exact(ws, st["emask"], N, M, objective=st["eobj"], workspace=wsp, stream=stream)
        tm.tmask_apply_pack(ws, st["emask"], st["packed"], N, M, stream=stream)
        tm.tmask_approx_pack(ws, None, st["fpacked"], N, M, stream=stream)
        tm.tmask_approx_dense(ws, None, st["dense"], N, M, stream=stream)

    def snapshot(st):
        out = [m.clone() for m in st["amask"] + st["emask"] + st["dense"]] + [st["aobj"].clone(), st["eobj"].clone()]
        for pk in st["packed"] + st["fpacked"]:
            out += [t.clone() for t in pk]
        return out

    eager = state()
    step(eager)
    torch.cuda.synchronize()
    want = snapshot(eager)
    st = state()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(st)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        step(st)
    for rep in range(3):
        for m in st["amask"] + st["emask"]:
            m.fill_(0x5A)
        for t in st["dense"]:
            t.fill_(9.0)
        for pk in st["packed"] + st["fpacked"]:
            for t in pk:
                t.view(torch.uint8).fill_(0xEE)
        junk = torch.randn(1 << 20, device="cuda").sum()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = snapshot(st)
        for a, b in zip(got, want):
            assert np.array_equal(a.cpu().numpy().view(np.uint8), b.cpu().numpy().view(np.uint8)), rep
        del junk


def test_m32_noalloc_and_counters_in_a_graph_replay_exactly():
    """What the first two tests leave out, recorded into one graph: the column-per-lane kernels (16:32: threshold form,
    priced start, staged pack, score), tmask_approx_noalloc (the entry point made for capture: nothing is allocated, the
    partial sums sit in the library's own array), and the two counting calls, whose counters are cleared by kernels."""
    N, M = 16, 32
    shapes = [(64, 128), (96, 416), (256, 1024)]
    ws = [torch.from_numpy(wl.gaussian_f32(r, c, seed=8200 + k, std=0.05)).cuda() for k, (r, c) in enumerate(shapes)]
    n = len(ws)
    wsp = tm.alloc_workspace(ws, N, M)

    def state():
        return {"amask": tm.alloc_masks(ws), "nmask": tm.alloc_masks(ws), "emask": tm.alloc_masks(ws),
                "aobj": torch.zeros(n, dtype=torch.float64, device="cuda"),
                "nobj": torch.zeros(n, dtype=torch.float64, device="cuda"),
                "eobj": torch.zeros(n, dtype=torch.float64, device="cuda"),
                "packed": [tm.alloc_packed(w, N, M) for w in ws],
                "sout": torch.zeros(n * tm.SCORE_OUT_BYTES, dtype=torch.uint8, device="cuda"),
                "flips": torch.zeros(n, dtype=torch.int64, device="cuda"),
                "viol": torch.zeros(n, dtype=torch.int64, device="cuda")}

    def step(st, stream=None):
        tm.tmask_approx(ws, st["amask"], N, M, objective=st["aobj"], workspace=wsp, stream=stream)
        tm.tmask_approx_noalloc(ws, st["nmask"], N, M, objective=st["nobj"], stream=stream)
        tm.tmask_exact(ws, st["emask"], N, M, objective=st["eobj"], workspace=wsp, stream=stream)
        tm.tmask_apply_pack(ws, st["emask"], st["packed"], N, M, stream=stream)
        tm.tmask_score(ws, st["emask"], N, M, st["sout"], workspace=wsp, stream=stream)
        tm.tmask_flip_count(st["amask"], st["emask"], [w.shape[1] for w in ws], st["flips"], stream=stream)
        tm.tmask_pattern_violations(ws, st["emask"], st["viol"], stream=stream)

    def snapshot(st):
        out = [m.clone() for m in st["amask"] + st["nmask"] + st["emask"]]
        out += [st[k].clone() for k in ("aobj", "nobj", "eobj", "sout", "flips", "viol")]
        for pk in st["packed"]:
            out += [t.clone() for t in pk]
        return out

    eager = state()
    step(eager)
    torch.cuda.synchronize()
    want = snapshot(eager)
    assert all(np.array_equal(a.cpu().numpy(), b.cpu().numpy()) for a, b in zip(eager["amask"], eager["nmask"]))
    assert int(eager["flips"].sum()) > 0 and int(eager["viol"].sum()) > 0
    st = state()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(st)                                  # warm-up on the capture stream (also looks up the library's array)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        step(st)
    for rep in range(3):
        for m in st["amask"] + st["nmask"] + st["emask"]:
            m.fill_(0x5A)
        for k in ("aobj", "nobj", "eobj"):
            st[k].fill_(-1.0)
        st["flips"].fill_(-7)
        st["viol"].fill_(-7)
        for pk in st["packed"]:
            for t in pk:
                t.view(torch.uint8).fill_(0xEE)
        junk = torch.randn(1 << 20, device="cuda").sum()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = snapshot(st)
        for a, b in zip(got, want):
            assert np.array_equal(a.cpu().numpy().view(np.uint8), b.cpu().numpy().view(np.uint8)), rep
        del junk

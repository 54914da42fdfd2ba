"""The sorting networks of the device code, read from the header as lists of wire indices and run here on every
zero-one input: a network of sorters (compare-exchanges, three-key sorts) that sorts those sorts everything."""
import itertools
import os
import re

import numpy as np

HEADER = os.path.join(os.path.dirname(__file__), "..", "paper_2102_08124_amd", "csrc", "tmask_networks.hpp")


def _body(n, name=None):
    src = open(HEADER).read()
    m = re.search(r"void %s\(uint32_t \(&v\)\[%d\]\)\s*\{(.*?)\n\}" % (name or "sort_asc<%d>" % n, n), src, re.S)
    assert m, "%s not found" % (name or "sort_asc<%d>" % n)
    return m.group(1)


def _ops(body):
    """[(i, j, k) | (i, j)] in program order."""
    out = []
    for name, args in re.findall(r"\b(sort3|cmpx)\(([^;]*?)\);", body):
        idx = tuple(int(x) for x in re.findall(r"v\[(\d+)\]", args))
        assert len(idx) == (3 if name == "sort3" else 2) and list(idx) == sorted(set(idx)), (name, args)
        out.append(idx)
    return out


def _run(ops, v):
    """v: (cases, wires) array; each op sorts its wires ascending in wire order."""
    v = v.copy()
    for idx in ops:
        v[:, list(idx)] = np.sort(v[:, list(idx)], axis=1)
    return v


def _zero_one(n):
    return np.array(list(itertools.product((0, 1), repeat=n)), dtype=np.uint8)


def test_sort4_and_sort8_sort_every_zero_one_input():
    for n, cost in ((4, 8), (8, 24)):
        ops = _ops(_body(n))
        assert sum(3 if len(o) == 3 else 2 for o in ops) == cost        # instruction count the comments state
        v = _zero_one(n)
        assert np.array_equal(_run(ops, v), np.sort(v, axis=1))


def test_sort16_sorts_every_zero_one_input_and_random_keys_with_repeats():
    body = _body(16)
    assert body.count("sort_asc<8>(") == 2 and body.count("merge_sorted8_asc(v)") == 1   # both halves, then the merge
    assert body.index("merge_sorted8_asc(v)") > body.rindex("sort_asc<8>(")
    merge = _ops(_body(16, "merge_sorted8_asc"))
    assert sum(3 if len(o) == 3 else 2 for o in merge) == 43
    sort8 = _ops(_body(8))
    halves = sort8 + [tuple(i + 8 for i in o) for o in sort8]
    v = _zero_one(16)
    assert np.array_equal(_run(halves + merge, v), np.sort(v, axis=1))
    rng = np.random.default_rng(5)
    for hi in (2, 3, 7, 1 << 31):
        r = rng.integers(0, hi, size=(20000, 16), dtype=np.int64)
        assert np.array_equal(_run(halves + merge, r), np.sort(r, axis=1))

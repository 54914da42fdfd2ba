"""Host-side checks of bench.py: the byte counts behind every roofline fraction, the traffic parser, and the refusal
of more than one GPU.  No GPU needed."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402


def test_algorithmic_bytes_per_weight():
    # bytes per weight of each call: s for W, 1 (or 1/8) for the mask, the packed operands 2 * (N/M) * (s + log2(M)/8),
    # 4 / M^2 for per-block objectives; per-matrix scalars on top
    W = 1 << 20
    for es in (4, 2):
        for (N, M) in ((2, 4), (4, 8), (8, 16), (16, 32), (3, 8)):
            b = bench.algorithmic_bytes(W, 0, es, N, M)
            ib = {4: 2, 8: 3, 16: 4, 32: 5}[M]
            packed = 2 * N / M * (es + ib / 8)
            assert b["approx"] / W == es + 1
            assert b["exact"] == b["approx"] == b["prune1d"]
            assert abs(b["pack"] / W - (es + 1 + packed)) < 1e-9
            assert abs(b["score"] / W - (es + 1 + 4 / (M * M))) < 1e-9
            assert abs(b["approx_pack"] / W - (es + packed)) < 1e-9
            assert b["approx_dense"] / W == 2 * es
            bits = bench.algorithmic_bytes(W, 0, es, N, M, bit_masks=True)
            assert bits["approx"] / W == es + 1 / 8
    # the figures quoted for the headline set (bf16, U8 masks, 2:4) and for fp32 2:4
    b = bench.algorithmic_bytes(W, 0, 2, 2, 4)
    assert (b["approx"] / W, b["score"] / W, b["pack"] / W) == (3.0, 3.25, 5.25)
    assert bench.algorithmic_bytes(W, 0, 4, 2, 4)["pack"] / W == 9.25
    # per-matrix scalars: one fp64 objective, one score record
    assert bench.algorithmic_bytes(W, 7, 2, 2, 4)["approx"] - b["approx"] == 7 * 8
    assert bench.algorithmic_bytes(W, 7, 2, 2, 4)["score"] - b["score"] == 7 * 56


def test_roofline_helper_and_peak():
    r = bench.hbm(8_000_000_000, 1000.0)          # 8 GB in one second
    assert r["achieved_GBs"] == 8.0 and abs(r["frac"] - 0.001) < 1e-12
    assert bench.HBM_PEAK_GBS == 8000.0


def test_traffic_parser_reads_the_committed_summary(tmp_path):
    p = tmp_path / "t.md"
    p.write_text("# x\n\n    traffic approx fetch_bytes=100 write_bytes=23\n    traffic pack fetch_bytes=5 write_bytes=7\nnoise\n")
    assert bench.read_pmc_traffic(str(p)) == {"approx": 123, "pack": 12}
    assert bench.read_pmc_traffic(str(tmp_path / "missing.md")) == {}
    got = bench.read_pmc_traffic(os.path.join(ROOT, "profiles", "pmc_traffic_bert_large_bf16_2of4.md"))
    assert set(got) == {"approx", "exact", "pack", "score"}
    alg = bench.algorithmic_bytes(301989888, 144, 2, 2, 4)
    for k, v in got.items():
        assert 0.98 < v / alg[k] < 1.05, (k, v / alg[k])      # measured traffic = what the method must move


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "--gpus 1" in r.stderr

#!/usr/bin/env python3
"""Timing of tmask_spmm24 (product with a packed 2:4 operand) on layer shapes, next to the dense library product.

    python -m paper_2102_08124_amd.sweep_spmm [--tokens 8192] [--shapes 4096x1024,1024x4096,1024x1024] [--reps 20]

Each line: kernel time from hipEvents around the kernel (marker overhead removed), dense-equivalent TFLOP/s
(2 * tokens * rows * cols / time) and its fraction of the 2.5 PFLOP/s dense bf16 peak, then the time of
torch's dense bf16 product of the same shape (x @ W^T with W expanded) for context.  A measuring aid.
"""
from __future__ import annotations

import argparse

import numpy as np
import torch

from . import binding as tm
from .hipevents import HipEvents

PEAK_TFLOPS = 2500.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--tokens", type=int, default=8192)
    ap.add_argument("--shapes", default="4096x1024,1024x4096,1024x1024,8192x8192")
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--out", default="f32", choices=["f32", "bf16"])
    a = ap.parse_args()
    ev = HipEvents()
    ovh = ev.empty_bracket_ms(torch.cuda.current_stream().cuda_stream)
    print("tokens %d, event overhead %.2f us" % (a.tokens, ovh * 1e3), flush=True)
    for shp in a.shapes.split(","):
        rows, cols = (int(v) for v in shp.split("x"))
        w = (torch.randn((rows, cols), device="cuda") * 0.02).to(torch.bfloat16)
        pk = tm.alloc_packed(w, 2, 4)
        tm.tmask_approx_pack([w], None, [pk], 2, 4)
        nb = 3
        xs = [torch.randn((a.tokens, cols), device="cuda").to(torch.bfloat16) for _ in range(nb)]
        odt = torch.float32 if a.out == "f32" else torch.bfloat16
        ys = [torch.empty((a.tokens, rows), dtype=odt, device="cuda") for _ in range(nb)]
        for k in range(nb):
            tm.tmask_spmm24(pk[0], pk[1], rows, cols, xs[k], ys[k])
        torch.cuda.synchronize()
        evs = [(ev.create(), ev.create()) for _ in range(a.reps)]
        for k in range(a.reps):
            tm.tmask_profile_next(*evs[k])
            tm.tmask_spmm24(pk[0], pk[1], rows, cols, xs[k % nb], ys[k % nb])
        torch.cuda.synchronize()
        ms = float(np.median([ev.elapsed_ms(*e) for e in evs])) - ovh
        flop = 2.0 * a.tokens * rows * cols
        # dense library product of the same shape (context only)
        wd = w.clone()
        yd = [torch.empty((a.tokens, rows), dtype=torch.bfloat16, device="cuda") for _ in range(nb)]
        for k in range(nb):
            torch.matmul(xs[k], wd.t(), out=yd[k])
        torch.cuda.synchronize()
        tev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(a.reps)]
        for k, (s, e) in enumerate(tev):
            s.record()
            torch.matmul(xs[k % nb], wd.t(), out=yd[k % nb])
            e.record()
        torch.cuda.synchronize()
        dms = float(np.median([s.elapsed_time(e) for s, e in tev]))
        print("spmm24 %5dx%-5d tokens %d out %s: %8.1f us  %7.1f TFLOP/s dense-equivalent  %4.1f%% of 2.5 PFLOP/s | "
              "torch dense bf16: %8.1f us  %7.1f TFLOP/s" % (rows, cols, a.tokens, a.out, ms * 1e3, flop / ms / 1e9,
                                                            flop / ms / 1e9 / PEAK_TFLOPS * 100, dms * 1e3, flop / dms / 1e9),
              flush=True)


if __name__ == "__main__":
    main()

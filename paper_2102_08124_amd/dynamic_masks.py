#!/usr/bin/env python3
"""Dynamic-mask surrogate of a training loop (the mask is extracted again as the weights move, Sec. 4.1):

    W_0 ~ N(0, 0.02) in bf16, W_t = W_{t-1} + 1e-3 * N(0, 0.02); every step recomputes the 2:4 transposable
    mask of W_t with tmask_approx and counts the entries that changed state against step t-1 with
    tmask_flip_count.

    python -m paper_2102_08124_amd.dynamic_masks [--side 16384] [--steps 200] [--fmt 0|1]

The weight update is input generation (torch, on the device); the mask and the flip count run in the library.
Prints the mean / last flip fraction and the steady-state rates of the mask kernel alone and of mask + count.
"""
from __future__ import annotations

import argparse

import numpy as np
import torch

from . import binding as tm
from .hipevents import HipEvents


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--side", type=int, default=16384)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--fmt", type=int, default=0, help="0 = U8 masks, 1 = BITS masks")
    a = ap.parse_args()
    side, T = a.side, a.side * a.side
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    w = (torch.randn((side, side), device="cuda", generator=gen) * 0.02).to(torch.bfloat16)
    noise = torch.empty((side, side), device="cuda", dtype=torch.float32)
    masks = [tm.alloc_masks([w], a.fmt)[0] for _ in range(2)]
    batches = [tm.MatBatch([w], [m]) for m in masks]
    flips = torch.zeros(a.steps + 1, dtype=torch.int64, device="cuda")
    ev = HipEvents()
    st = torch.cuda.current_stream().cuda_stream
    ovh = ev.empty_bracket_ms(st)
    tm.tmask_approx(batches[0], None, 2, 4, mask_fmt=a.fmt)
    t_mask, t_both = [], []
    for t in range(1, a.steps + 1):
        noise.normal_(0.0, 0.02 * 1e-3, generator=gen)
        w.add_(noise.to(torch.bfloat16))
        e0, e1, e2 = ev.create(), ev.create(), ev.create()
        ev.record(e0, st)
        tm.tmask_approx(batches[t & 1], None, 2, 4, mask_fmt=a.fmt)
        ev.record(e1, st)
        tm.tmask_flip_count([masks[t & 1]], [masks[(t - 1) & 1]], [side], flips[t:t + 1], mask_fmt=a.fmt)
        ev.record(e2, st)
        torch.cuda.synchronize()
        t_mask.append(ev.elapsed_ms(e0, e1) - ovh)
        t_both.append(ev.elapsed_ms(e0, e2) - ovh)
    frac = flips[1:].cpu().numpy() / float(T)
    half = a.steps // 2
    ms_mask, ms_both = float(np.median(t_mask[half:])), float(np.median(t_both[half:]))
    print("side %d bf16, %d steps, %s masks" % (side, a.steps, "BITS" if a.fmt else "U8"))
    print("flip fraction per step: mean %.5f, first %.5f, last %.5f" % (frac.mean(), frac[0], frac[-1]))
    print("mask kernel: %.1f us per step, %.3e weights/s" % (ms_mask * 1e3, T / ms_mask * 1e3))
    print("mask + flip count: %.1f us per step, %.3e weights/s" % (ms_both * 1e3, T / ms_both * 1e3))


if __name__ == "__main__":
    main()

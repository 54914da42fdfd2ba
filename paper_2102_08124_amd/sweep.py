#!/usr/bin/env python3
"""Per-kernel timing of the four entry points over dtype x N:M on one square matrix.

    python -m paper_2102_08124_amd.sweep [--side 8192] [--calls approx,exact,score,pack,fused,fusedm,prune1d,flip,dense,absorb,adense,p1dense,p1absorb,viol] [--dts f32,bf16] [--ms 4,8,16]

Each line: main-kernel time from hipEvents recorded around the kernel (marker overhead removed),
algorithmic GB/s, fraction of the 8 TB/s HBM peak, weights/s.  Inputs are N(0, 0.02) generated on the
device; three buffer sets are rotated.  This is a measuring aid, not part of the method.
"""
from __future__ import annotations

import argparse

import numpy as np
import torch

from . import binding as tm
from .hipevents import HipEvents


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--side", type=int, default=8192)
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--calls", default="approx,exact,score,pack")
    ap.add_argument("--dts", default="f32,bf16")
    ap.add_argument("--ms", default="4,8,16")
    ap.add_argument("--fmt", type=int, default=0, help="0 = U8 masks, 1 = BITS masks")
    a = ap.parse_args()
    ev = HipEvents()
    ovh = ev.empty_bracket_ms(torch.cuda.current_stream().cuda_stream)
    side = a.side
    print("side %d, event overhead %.2f us" % (side, ovh * 1e3), flush=True)
    for dt in a.dts.split(","):
        nb = 3
        ws = [(torch.randn((side, side), device="cuda") * 0.02).to(torch.float32 if dt == "f32" else torch.bfloat16)
              for _ in range(nb)]
        es = 4 if dt == "f32" else 2
        for M in [int(x) for x in a.ms.split(",")]:
            N = M // 2
            masks = [tm.alloc_masks([w], a.fmt)[0] for w in ws]
            obj = torch.zeros(1, dtype=torch.float64, device="cuda")
            wsp = tm.alloc_workspace([ws[0]], N, M)
            sout = torch.zeros(tm.SCORE_OUT_BYTES, dtype=torch.uint8, device="cuda")
            pb = torch.zeros(side * side // (M * M), dtype=torch.float32, device="cuda")
            # outputs rotate like the inputs: a buffer rewritten by every call would partly stay in the
            # memory-side cache and flatter kernels whose stores allocate there
            packeds = [tm.alloc_packed(ws[0], N, M) for _ in range(nb)]
            flips = torch.zeros(1, dtype=torch.int64, device="cuda")
            dense_outs = [torch.empty_like(ws[0]) for _ in range(nb)]
            viol_count = torch.zeros(1, dtype=torch.int64, device="cuda")
            T = side * side
            mb = T if a.fmt == 0 else T // 8
            ib = (M - 1).bit_length()
            byts = {"approx": T * es + mb, "exact": T * es + mb, "score": T * es + mb + 4 * T // (M * M),
                    "pack": T * es + mb + 2 * (T * N // M) * es + 2 * (T * N // M) * ib // 8,
                    "prune1d": T * es + mb, "flip": 2 * mb, "dense": 2 * T * es + mb, "absorb": 2 * T * es + mb, "adense": 2 * T * es, "p1dense": 2 * T * es, "p1absorb": 2 * T * es, "viol": T * es + mb,
                    "fused": T * es + 2 * (T * N // M) * es + 2 * (T * N // M) * ib // 8,
                    "fusedm": T * es + mb + 2 * (T * N // M) * es + 2 * (T * N // M) * ib // 8}
            for call in a.calls.split(","):
                def run(k):
                    w, m, packed, dense_out = ws[k % nb], masks[k % nb], packeds[k % nb], dense_outs[k % nb]
                    if call == "approx":
                        tm.tmask_approx([w], [m], N, M, objective=obj, mask_fmt=a.fmt, workspace=wsp)
                    elif call == "exact":
                        tm.tmask_exact([w], [m], N, M, objective=obj, mask_fmt=a.fmt, workspace=wsp)
                    elif call == "score":
                        tm.tmask_score([w], [m], N, M, sout, per_block_obj=pb, mask_fmt=a.fmt, workspace=wsp)
                    elif call == "prune1d":
                        tm.tmask_prune_1d([w], [m], N, M, objective=obj, mask_fmt=a.fmt, workspace=wsp)
                    elif call == "flip":
                        tm.tmask_flip_count([m], [masks[(k + 1) % nb]], [side], flips, mask_fmt=a.fmt)
                    elif call in ("dense", "absorb"):   # masked copy, without / with mean absorption
                        tm.tmask_apply_dense([w], [m], [dense_out], M, call == "absorb", mask_fmt=a.fmt)
                    elif call == "adense":              # Algorithm 1 + masked copy in one pass, no mask written
                        tm.tmask_approx_dense([w], None, [dense_out], N, M, mask_fmt=a.fmt)
                    elif call == "viol":                # pattern violations: non-zero weights the mask removes
                        tm.tmask_pattern_violations([w], [m], viol_count, mask_fmt=a.fmt)
                    elif call in ("p1dense", "p1absorb"):   # row pruning + masked copy (+ mean absorption), no mask written
                        tm.tmask_prune_1d_dense([w], None, [dense_out], N, M, call == "p1absorb", mask_fmt=a.fmt)
                    elif call == "fused":      # Algorithm 1 + compression in one call, no mask written (2:4 only)
                        tm.tmask_approx_pack([w], None, [packed], N, M, mask_fmt=a.fmt)
                    elif call == "fusedm":     # the same with the mask written too
                        tm.tmask_approx_pack([w], [m], [packed], N, M, mask_fmt=a.fmt)
                    else:
                        tm.tmask_apply_pack([w], [m], [packed], N, M, mask_fmt=a.fmt)
                if call in ("score", "pack", "flip", "dense", "absorb", "viol"):
                    for k in range(nb):
                        tm.tmask_approx([ws[k]], [masks[k]], N, M, mask_fmt=a.fmt)
                run(0)
                run(1)
                torch.cuda.synchronize()
                evs = [(ev.create(), ev.create()) for _ in range(a.reps)]
                for k in range(a.reps):
                    tm.tmask_profile_next(*evs[k])
                    run(k)
                torch.cuda.synchronize()
                ms = float(np.median([ev.elapsed_ms(*e) for e in evs])) - ovh
                print("%-6s %-4s %d:%-2d  %8.1f us  %7.1f GB/s  %5.1f%% of 8TB/s  %7.1f Gweights/s" %
                      (call, dt, N, M, ms * 1e3, byts[call] / ms / 1e6, byts[call] / ms / 1e6 / 80, T / ms / 1e6),
                      flush=True)
        del ws


if __name__ == "__main__":
    main()

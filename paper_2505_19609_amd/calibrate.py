"""Offline profiling for the paper's latency model T_comp = alpha * FLOPs + beta
(App. B.2): time this library's forward + backward on single whole sequences over a range
of lengths and fit alpha, beta by least squares against the attention term of FLOPs(S),
4*b*h*S^2 (the part of the layer this library computes).  Also times the 1/N share
of each length that DACP's FLOPs(S)/N stands for (Eq. 4), for the first and the last rank under
both cuts (contiguous slice, two balanced chunks).

    python -m paper_2505_19609_amd.calibrate --model qwen2.5-7b --cp 8
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np

from .dacp_run import run_rank


def main(argv=None):
    from . import workloads as W
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--model", choices=sorted(W.MODEL_SHAPES), default="qwen2.5-0.5b")
    ap.add_argument("--cp", type=int, default=8)
    ap.add_argument("--lengths", type=int, nargs="*",
                    default=[256, 512, 1024, 2048, 4096, 8192, 16384, 32768, 65536])
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args(argv)

    import torch
    if not torch.cuda.is_available():
        print("calibrate: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    h, hkv, hq, hk, d = W.MODEL_SHAPES[args.model]
    rows = []
    for L in args.lengths:
        whole, info = run_rank([L], [1], [0], (hq, hk), d, args.reps, L)
        row = {"S": L, "attn_flops_model": 4 * h * L * L, "whole_ms": round(whole, 4),
               "whole_useful_tflops": round(info["useful_flops"] / (whole * 1e-3) / 1e12, 1)}
        if L >= 2 * args.cp:
            first, _ = run_rank([L], [args.cp], [0], (hq, hk), d, args.reps, L + 1)
            last, _ = run_rank([L], [args.cp], [args.cp - 1], (hq, hk), d, args.reps, L + 2)
            two0, _ = run_rank([L], [args.cp], [0], (hq, hk), d, args.reps, L + 3, cut=1)
            two1, _ = run_rank([L], [args.cp], [args.cp - 1], (hq, hk), d, args.reps, L + 4, cut=1)
            row.update(slice_first_ms=round(first, 4), slice_last_ms=round(last, 4),
                       two_chunks_first_ms=round(two0, 4), two_chunks_last_ms=round(two1, 4))
        rows.append(row)
    x = np.array([r["attn_flops_model"] for r in rows], np.float64)
    y = np.array([r["whole_ms"] for r in rows], np.float64)
    A = np.stack([x, np.ones_like(x)], 1)
    (alpha, beta), *_ = np.linalg.lstsq(A, y, rcond=None)
    resid = y - A @ np.array([alpha, beta])
    r2 = 1.0 - float(resid @ resid) / float(((y - y.mean()) ** 2).sum())
    print(json.dumps({"model": args.model, "cp_degree": args.cp, "fit": "whole_ms = alpha * 4*h*S^2 + beta",
                      "alpha_ms_per_flop": alpha, "beta_ms": round(float(beta), 4), "r2": round(r2, 5),
                      "rows": rows}))
    return 0


if __name__ == "__main__":
    sys.exit(main())

"""Measurements behind the plan's launch-shape rules: the same micro-batch timed with each
choice forced, next to the choice the plan makes by itself.

    python -m paper_2505_19609_amd.shape_sweep wg     # forward / dQ workgroup of 128 or 256 query rows
    python -m paper_2505_19609_amd.shape_sweep dkv    # dK/dV items of 128 or 192 key rows (head_dim 64), head split

One line per (head shape, length mix): kernel times in ms (median of HIP events over the
repetitions) for every forced choice, and what `skrull_attn_plan` picks when the field is left 0.
"""
from __future__ import annotations

import argparse
import sys

import numpy as np

MIXES = {
    "128x256": [256] * 128, "64x512": [512] * 64, "32x1024": [1024] * 32, "16x2048": [2048] * 16,
    "8x4096": [4096] * 8, "4x8192": [8192] * 4, "2x16384": [16384] * 2, "1x32768": [32768],
    "6000+26x1024": [6000] + [1024] * 26, "24576+8x1024": [24576] + [1024] * 8,
    "ragged": [5000, 3001, 777, 129, 64, 12000, 33, 2049],
}


def _mixes():
    from . import workloads as W
    rng = np.random.Generator(np.random.PCG64(5))
    logn = [int(x) for x in np.clip(np.round(np.exp(rng.normal(np.log(900), 0.9, 40))), 32, 6000)]
    return {"config2": list(W.config(2).seq_len), "config2x2": list(W.config(2).seq_len) * 2, "lognormal40": logn, **MIXES}


def _time(S, heads, d, reps, **plan_args):
    """(fwd, dq, dkv) ms and the plan's info for one forced choice."""
    import torch
    from . import binding as B
    hq, hkv = heads
    plan = B.skrull_attn_plan(S, [1] * len(S), [0] * len(S), hq, hkv, d, d ** -0.5, **plan_args)
    gen = torch.Generator(device="cuda").manual_seed(1)
    rnd = lambda rows, h: torch.randn((rows, h, d), generator=gen, device="cuda").bfloat16()  # noqa: E731
    q, k, v, do = rnd(plan.total_q, hq), rnd(plan.total_k, hkv), rnd(plan.total_k, hkv), rnd(plan.total_q, hq)
    o, dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    lse = torch.empty((hq, plan.total_q), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(int(plan.bwd_workspace_bytes), 16), dtype=torch.uint8, device="cuda")

    def step():
        B.skrull_attn_fwd(plan, q, k, v, o, lse)
        B.skrull_attn_bwd(plan, q, k, v, o, lse, do, dq, dk, dv, ws)

    for _ in range(2):
        step()
    torch.cuda.synchronize()
    B.skrull_attn_profile(True)
    ms = np.zeros((reps, 4))
    for i in range(reps):
        step()
        ms[i] = B.skrull_attn_profile_read()
    B.skrull_attn_profile(False)
    m = np.median(ms, axis=0)
    info = plan.info
    picked = (int(info.wg_query_rows), int(info.block_n), int(info.head_split))
    plan.destroy()
    return (m[0], m[3], m[2]), picked


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("what", choices=("wg", "dkv"))
    ap.add_argument("--reps", type=int, default=9)
    args = ap.parse_args(argv)
    import torch
    if not torch.cuda.is_available():
        print("shape_sweep: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    mixes = _mixes()
    if args.what == "wg":
        shapes = [((8, 2), 128), ((16, 4), 128), ((28, 4), 128), ((32, 8), 128), ((64, 8), 128),
                  ((8, 8), 64), ((14, 2), 64), ((16, 16), 64), ((32, 8), 64), ((64, 8), 64)]
        names = ["config2", "128x256", "32x1024", "16x2048", "8x4096", "4x8192", "2x16384", "1x32768", "6000+26x1024", "ragged"]
        print("heads/head_dim mix: forward ms with 128 / 256 query rows per workgroup (128 against 256), dQ likewise; plan picks")
        for heads, d in shapes:
            for n in names:
                (f1, q1, _), _ = _time(mixes[n], heads, d, args.reps, wg_query_rows=128)
                (f2, q2, _), _ = _time(mixes[n], heads, d, args.reps, wg_query_rows=256)
                _, picked = _time(mixes[n], heads, d, 1)
                print(f"{heads[0]}/{heads[1]}/{d} {n}: fwd {f1:.3f} / {f2:.3f} ({100 * (f1 / f2 - 1):+.1f} %)  "
                      f"dQ {q1:.3f} / {q2:.3f} ({100 * (q1 / q2 - 1):+.1f} %)  plan picks {picked[0]}", flush=True)
    else:
        shapes = [((14, 2), 64), ((32, 4), 64), ((32, 8), 64), ((16, 16), 64), ((64, 8), 64),
                  ((16, 1), 128), ((32, 2), 128), ((28, 4), 128), ((32, 8), 128)]
        names = ["config2", "config2x2", "lognormal40", "128x256", "64x512", "32x1024", "8x4096", "4x8192", "1x32768",
                 "6000+26x1024", "24576+8x1024", "ragged"]
        print("heads/head_dim mix: dK/dV ms for block_n/head_split forced; plan picks")
        for heads, d in shapes:
            g = heads[0] // heads[1]
            splits = sorted({1, g} | {x for x in (2, 4, 8) if g % x == 0 and x <= g})
            blocks = (128, 192) if d == 64 else (128,)
            for n in names:
                cells = []
                for bn in blocks:
                    for hs in splits:
                        (_, _, t), _ = _time(mixes[n], heads, d, args.reps, block_n=bn, head_split=hs)
                        cells.append(f"{bn}/{hs} {t:.3f}")
                (_, _, t), picked = _time(mixes[n], heads, d, args.reps)
                print(f"{heads[0]}/{heads[1]}/{d} {n}: " + "  ".join(cells) + f"  plan picks {picked[1]}/{picked[2]} {t:.3f}", flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())

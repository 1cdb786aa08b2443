"""Schedule one micro-batch with DACP and run every context-parallel rank's share of
it on this one GPU, one rank after another.

The paper's objective (Sec. 4.1, Eq. 1) is the time of the slowest rank,
max_j Time_j; its heuristic (Sec. 4.3.2, Alg. 1) balances the FLOPs-model load of the
ranks.  This driver measures the attention part of Time_j directly: for each rank j
it builds the rank's micro-batch from the schedule (local sequences whole, slice j of
every distributed one), runs the library's forward + backward on it and reports the
per-rank times, their maximum and minimum, and the time the scheduler itself took.
With --compare it also runs the same sequences under plain context parallelism
(every sequence cut over all N ranks), the paper's baseline.

Every step of the attention path runs in the HIP library; the schedule comes from the
library's host scheduler.  Communication (Eq. 2-3) is not modelled: this is one GPU.

    python -m paper_2505_19609_amd.dacp_run --dataset chatqa2_long_sft \
        --model qwen2.5-0.5b --cp 8 --bucket 26624
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np


def draw_micro_batch(dataset: str, bucket: int, cp: int, fill: float, seed: int):
    """Sequence lengths from the Table 1 mix of `dataset` up to fill*C*N tokens, no
    sequence longer than the C*N tokens a micro-batch can hold at all."""
    from . import workloads as W
    rng = np.random.Generator(np.random.PCG64(seed))
    return W.table1_lengths(rng, dataset, budget=int(fill * bucket * cp), longest=bucket * cp)


def run_rank(seq_len, degree, index, heads, head_dim, reps: int, seed: int, cut: int = 0):
    """Forward + backward of one rank's micro-batch; returns (ms per fwd+bwd, plan totals).
    `cut` is how distributed sequences are cut (0 contiguous slice, 1 two balanced chunks)."""
    import torch
    from . import binding as B

    hq, hkv = heads
    shard_cut = [cut if n > 1 else 0 for n in degree]
    plan = B.skrull_attn_plan(seq_len, degree, index, hq, hkv, head_dim, head_dim ** -0.5,
                              shard_cut=shard_cut)
    tq, tk = plan.total_q, plan.total_k
    gen = torch.Generator(device="cuda").manual_seed(seed)

    def rnd(rows, h):
        return torch.randn((rows, h, head_dim), generator=gen, device="cuda", dtype=torch.float32).bfloat16()

    q, k, v, do = rnd(tq, hq), rnd(tk, hkv), rnd(tk, hkv), rnd(tq, hq)
    o, dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    lse = torch.empty((hq, tq), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(int(plan.bwd_workspace_bytes), 16), dtype=torch.uint8, device="cuda")

    def once():
        B.skrull_attn_fwd(plan, q, k, v, o, lse)
        B.skrull_attn_bwd(plan, q, k, v, o, lse, do, dq, dk, dv, ws)

    once()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        once()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / reps * 1e3
    info = {"tokens": int(tq), "kv_rows": int(tk),
            "useful_flops": int(plan.useful_flops_fwd + plan.useful_flops_bwd)}
    plan.destroy()
    return ms, info


def run_schedule(S, ret, cp: int, heads, head_dim: int, reps: int, seed: int, cut: int = 0):
    """Per-rank measurements of schedule `ret` (Alg. 1's output array)."""
    from . import binding as B
    ranks = []
    for j in range(cp):
        seq, deg, idx, _ = B.skrull_dacp_rank_batch(S, ret, cp, j)
        if len(seq) == 0:
            ranks.append({"rank": j, "tokens": 0, "kv_rows": 0, "useful_flops": 0, "ms": 0.0,
                          "local": 0, "distributed": 0})
            continue
        ms, info = run_rank(seq, deg, idx, heads, head_dim, reps, seed + j, cut)
        info.update(rank=j, ms=round(ms, 4), local=int((deg == 1).sum()), distributed=int((deg != 1).sum()))
        ranks.append(info)
    t = np.array([r["ms"] for r in ranks])
    fl = sum(r["useful_flops"] for r in ranks)
    return {"max_ms": round(float(t.max()), 4), "min_ms": round(float(t.min()), 4),
            "mean_ms": round(float(t.mean()), 4),
            "useful_tflops_at_max": round(fl / cp / (t.max() * 1e-3) / 1e12, 2) if t.max() > 0 else 0.0,
            "ranks": ranks}


def main(argv=None):
    from . import workloads as W
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--dataset", choices=sorted(W.TABLE1), default="chatqa2_long_sft")
    ap.add_argument("--model", choices=sorted(W.MODEL_SHAPES), default="qwen2.5-0.5b")
    ap.add_argument("--cp", type=int, default=8, help="context-parallel degree N")
    ap.add_argument("--bucket", type=int, default=26 * 1024, help="BucketSize C, tokens per rank")
    ap.add_argument("--fill", type=float, default=0.8, help="tokens drawn, as a share of C*N")
    ap.add_argument("--seq-len", type=int, nargs="*", help="explicit lengths instead of a drawn mix")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--compare", action="store_true", help="also run plain CP (every sequence distributed)")
    ap.add_argument("--cut", choices=["contiguous", "two-chunks"], default="two-chunks",
                    help="how a distributed sequence is cut over the ranks")
    args = ap.parse_args(argv)

    import torch
    from . import binding as B
    if not torch.cuda.is_available():
        print("dacp_run: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    h, hkv, hq, hk, d = W.MODEL_SHAPES[args.model]
    S = args.seq_len or draw_micro_batch(args.dataset, args.bucket, args.cp, args.fill, args.seed)
    cut = 1 if args.cut == "two-chunks" else 0
    S = [s for s in S if s >= (1 + cut) * args.cp]   # a sequence cannot be cut into more chunks than tokens

    sched_us = float("inf")
    for _ in range(5):   # best of five: the first call also pays for loading the library
        t0 = time.perf_counter()
        ret = B.skrull_dacp_schedule(S, args.bucket, args.cp, h, hkv)
        sched_us = min(sched_us, (time.perf_counter() - t0) * 1e6)
    out = {"dataset": "explicit" if args.seq_len else args.dataset, "model": args.model,
           "cp_degree": args.cp, "cut": args.cut, "bucket_size": args.bucket, "num_seqs": len(S), "tokens": int(sum(S)),
           "longest": int(max(S)), "schedule_us": round(sched_us, 1),
           "distributed_seqs": int((ret == -1).sum()), "local_seqs": int((ret != -1).sum()),
           "dacp": run_schedule(S, ret, args.cp, (hq, hk), d, args.reps, args.seed, cut)}
    if args.compare:
        plain = np.full(len(S), -1, np.int32)
        out["plain_cp"] = run_schedule(S, plain, args.cp, (hq, hk), d, args.reps, args.seed, cut)
        out["speedup_max_rank_time"] = round(out["plain_cp"]["max_ms"] / out["dacp"]["max_ms"], 3)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())

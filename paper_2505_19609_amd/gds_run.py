"""Schedule one training iteration's global batch with GDS + DACP and run it on this one
GPU: every micro-batch of one DP rank (or of all of them), every context-parallel rank's
share of each, one after another.

The paper's joint objective (Sec. 4.2) is max_i sum_j Time_ij with Time_ij the time of
the slowest CP rank on micro-batch j of DP rank i; this driver measures the attention
part of exactly that: sum over micro-batches of the slowest rank's forward + backward
time, per DP rank, and its maximum over the DP ranks that were run.  The global batch is
drawn from the Table 1 length mix of the named corpus with the paper's settings as
defaults (Sec. 5: BatchSize 64 per DP rank, DP 4, CP 8, BucketSize 26K).

    python -m paper_2505_19609_amd.gds_run --dataset chatqa2_long_sft --model qwen2.5-0.5b
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np

from .dacp_run import run_schedule


def main(argv=None):
    from . import workloads as W
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--dataset", choices=sorted(W.TABLE1), default="chatqa2_long_sft")
    ap.add_argument("--model", choices=sorted(W.MODEL_SHAPES), default="qwen2.5-0.5b")
    ap.add_argument("--cp", type=int, default=8, help="context-parallel degree N")
    ap.add_argument("--dp", type=int, default=4, help="DP world size ws")
    ap.add_argument("--dp-rank", type=int, default=None, help="run only this DP rank (default: all)")
    ap.add_argument("--batch-size", type=int, default=64, help="sequences per DP rank in the global batch")
    ap.add_argument("--bucket", type=int, default=26 * 1024, help="BucketSize C, tokens per CP rank")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--reps", type=int, default=2)
    ap.add_argument("--cut", choices=["contiguous", "two-chunks"], default="two-chunks",
                    help="how a distributed sequence is cut over the CP ranks")
    args = ap.parse_args(argv)

    import torch
    from . import binding as B
    if not torch.cuda.is_available():
        print("gds_run: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    h, hkv, hq, hk, d = W.MODEL_SHAPES[args.model]
    rng = np.random.Generator(np.random.PCG64(args.seed))
    cut = 1 if args.cut == "two-chunks" else 0
    # no sequence longer than a micro-batch can hold, none with fewer tokens than chunks
    S = [max(s, (1 + cut) * args.cp) for s in W.table1_lengths(rng, args.dataset, count=args.batch_size * args.dp,
                                                   longest=args.bucket * args.cp)]
    S = np.asarray(S, np.int32)
    out = {"dataset": args.dataset, "model": args.model, "cp_degree": args.cp, "cut": args.cut, "dp_world_size": args.dp,
           "bucket_size": args.bucket, "num_seqs": int(S.size), "tokens": int(S.sum()),
           "longest": int(S.max()), "dp_ranks": []}
    for r in ([args.dp_rank] if args.dp_rank is not None else range(args.dp)):
        sched_us = float("inf")
        for _ in range(3):
            t0 = time.perf_counter()
            bins, mb, ret, m = B.skrull_gds_schedule(S, args.bucket, args.cp, args.dp, r, h, hkv)
            sched_us = min(sched_us, (time.perf_counter() - t0) * 1e6)
        rank = {"dp_rank": r, "num_seqs": int((bins == r).sum()), "tokens": int(S[bins == r].sum()),
                "micro_batches": [], "schedule_us": round(sched_us, 1)}
        total = 0.0
        for j in range(m):
            members = B.skrull_gds_micro_batch(S, mb, j)
            res = run_schedule(S[members], ret[members], args.cp, (hq, hk), d, args.reps, args.seed + 100 * j, cut)
            total += res["max_ms"]
            rank["micro_batches"].append({"num_seqs": int(members.size), "tokens": int(S[members].sum()),
                                          "distributed": int((ret[members] == -1).sum()),
                                          "max_ms": res["max_ms"], "min_ms": res["min_ms"],
                                          "mean_ms": res["mean_ms"]})
        rank["sum_max_ms"] = round(total, 4)
        out["dp_ranks"].append(rank)
    out["iteration_ms"] = max(r["sum_max_ms"] for r in out["dp_ranks"])
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())

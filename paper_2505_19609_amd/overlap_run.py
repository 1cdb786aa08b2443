"""One CP rank's micro-batch with the exchange of its distributed sequences overlapped
with the attention of its local ones, on two HIP streams of this one GPU.

The paper's per-rank time (Sec. 4.1, Eq. 2) is
    max(T_comm(distributed), T_comp(local)) + T_comp(distributed):
local sequences need no exchange, so their attention hides the gather of the
distributed sequences' keys and values; the backward mirrors it (the partial dK/dV of
the distributed sequences leave while the local sequences' backward runs).  There is
one GPU here and no collective, so a plain copy stands in for each exchange: the
key/value rows of the prefix that live on OTHER ranks arrive from a staging buffer
(pinned host memory by default, so the copy engine moves them, as a link would; or a
second device buffer), and the partial dK/dV of those rows leave the same way.

The rank's micro-batch is planned as two plans, local and distributed; the attention
results are bit-identical to planning it as one (work items never mix sequences).
Streams keep the default priority.

    python -m paper_2505_19609_amd.overlap_run --seq-len 131072 --local-budget 8192 --model llama-3-8b
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np


class RankBatch:
    """Device tensors and plans of one rank's share: `loc` = whole sequences,
    `dist` = its slices of distributed ones."""

    def __init__(self, loc, dist, heads, head_dim, seed, source, head_split=0):
        import torch
        from . import binding as B
        self.B, self.torch = B, torch
        hq, hkv = heads
        gen = torch.Generator(device="cuda").manual_seed(seed)
        self.parts = {}
        for name, (S, deg, idx, cut) in (("loc", loc), ("dist", dist)):
            if len(S) == 0:
                self.parts[name] = None
                continue
            plan = B.skrull_attn_plan(S, deg, idx, hq, hkv, head_dim, head_dim ** -0.5, shard_cut=cut,
                                     head_split=head_split)
            tq, tk = plan.total_q, plan.total_k

            def rnd(rows, h):
                return torch.randn((rows, h, head_dim), generator=gen, device="cuda",
                                   dtype=torch.float32).bfloat16()

            t = {"plan": plan, "q": rnd(tq, hq), "k": rnd(tk, hkv), "v": rnd(tk, hkv), "do": rnd(tq, hq)}
            for n, like in (("o", "q"), ("dq", "q"), ("dk", "k"), ("dv", "k")):
                t[n] = torch.empty_like(t[like])
            t["lse"] = torch.empty((hq, tq), dtype=torch.float32, device="cuda")
            t["ws"] = torch.empty(max(int(plan.bwd_workspace_bytes), 16), dtype=torch.uint8, device="cuda")
            self.parts[name] = t
        d = self.parts["dist"]
        # rows of the distributed prefixes that other ranks own: what the gather brings in
        # and what the reduce-scatter of dK/dV sends out
        self.remote_rows = 0 if d is None else int(d["plan"].total_k - d["plan"].total_q)
        if self.remote_rows > 0:
            shape = (self.remote_rows, hkv, head_dim)
            if source == "host":
                mk = lambda: torch.empty(shape, dtype=torch.bfloat16).pin_memory()  # noqa: E731
            else:
                mk = lambda: torch.empty(shape, dtype=torch.bfloat16, device="cuda")  # noqa: E731
            self.stage = {n: mk() for n in ("k", "v", "dk", "dv")}
            self.stage["k"].copy_(d["k"][:self.remote_rows])
            self.stage["v"].copy_(d["v"][:self.remote_rows])
        self.comp = torch.cuda.Stream()
        self.comm = torch.cuda.Stream()

    # --- the five pieces -------------------------------------------------------------
    def gather(self):
        d = self.parts["dist"]
        if self.remote_rows > 0:
            d["k"][:self.remote_rows].copy_(self.stage["k"], non_blocking=True)
            d["v"][:self.remote_rows].copy_(self.stage["v"], non_blocking=True)

    def scatter(self):
        d = self.parts["dist"]
        if self.remote_rows > 0:
            self.stage["dk"].copy_(d["dk"][:self.remote_rows], non_blocking=True)
            self.stage["dv"].copy_(d["dv"][:self.remote_rows], non_blocking=True)

    def fwd(self, name):
        t = self.parts[name]
        if t is not None:
            self.B.skrull_attn_fwd(t["plan"], t["q"], t["k"], t["v"], t["o"], t["lse"])

    def bwd(self, name):
        t = self.parts[name]
        if t is not None:
            self.B.skrull_attn_bwd(t["plan"], t["q"], t["k"], t["v"], t["o"], t["lse"], t["do"],
                                   t["dq"], t["dk"], t["dv"], t["ws"])

    # --- two orders ------------------------------------------------------------------
    def step_serial(self):
        torch = self.torch
        with torch.cuda.stream(self.comp):
            self.gather()
            self.fwd("loc")
            self.fwd("dist")
            self.bwd("dist")
            self.scatter()
            self.bwd("loc")

    def step_overlapped(self):
        torch = self.torch
        arrived, partials_ready = torch.cuda.Event(), torch.cuda.Event()
        self.comm.wait_stream(self.comp)          # the previous step has let go of the buffers
        with torch.cuda.stream(self.comm):
            self.gather()
            arrived.record()
        with torch.cuda.stream(self.comp):
            self.fwd("loc")                       # hides the gather
            self.comp.wait_event(arrived)
            self.fwd("dist")
            self.bwd("dist")
            partials_ready.record()
        with torch.cuda.stream(self.comm):
            self.comm.wait_event(partials_ready)
            self.scatter()
        with torch.cuda.stream(self.comp):
            self.bwd("loc")                       # hides the scatter
            self.comp.wait_stream(self.comm)

    def outputs(self):
        out = {}
        for name, t in self.parts.items():
            if t is not None:
                for n in ("o", "lse", "dq", "dk", "dv"):
                    out[f"{name}.{n}"] = t[n].clone()
        if self.remote_rows > 0:
            out["stage.dk"], out["stage.dv"] = self.stage["dk"].clone(), self.stage["dv"].clone()
        return out

    def time_ms(self, fn, reps):
        torch = self.torch
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps * 1e3

    def destroy(self):
        for t in self.parts.values():
            if t is not None:
                t["plan"].destroy()


def main(argv=None):
    from . import workloads as W
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--model", choices=sorted(W.MODEL_SHAPES), default="llama-3-8b")
    ap.add_argument("--cp", type=int, default=8)
    ap.add_argument("--rank", type=int, default=None, help="CP rank to run (default: the last)")
    ap.add_argument("--seq-len", type=int, default=131072, help="the distributed sequence")
    ap.add_argument("--local-budget", type=int, default=8192, help="tokens of short local sequences")
    ap.add_argument("--cut", choices=["contiguous", "two-chunks"], default="two-chunks")
    ap.add_argument("--source", choices=["host", "device"], default="host",
                    help="where the stand-in for the exchanged rows lives")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args(argv)

    import torch
    if not torch.cuda.is_available():
        print("overlap_run: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    _, _, hq, hk, d = W.MODEL_SHAPES[args.model]
    rng = np.random.Generator(np.random.PCG64(args.seed))
    short = W.lognormal_lengths(rng, 1000, 0.8, 64, 4096, args.local_budget)
    r = args.cp - 1 if args.rank is None else args.rank
    cut = 1 if args.cut == "two-chunks" else 0
    loc = (short, [1] * len(short), [0] * len(short), [0] * len(short))
    dist = ([args.seq_len], [args.cp], [r], [cut])
    rb = RankBatch(loc, dist, (hq, hk), d, args.seed, args.source)
    pieces = {}
    for name, fn in (("gather", rb.gather), ("scatter", rb.scatter), ("fwd_local", lambda: rb.fwd("loc")),
                     ("fwd_dist", lambda: rb.fwd("dist")), ("bwd_local", lambda: rb.bwd("loc")),
                     ("bwd_dist", lambda: rb.bwd("dist"))):
        pieces[name] = round(rb.time_ms(fn, args.reps), 4)
    serial = rb.time_ms(rb.step_serial, args.reps)
    overlapped = rb.time_ms(rb.step_overlapped, args.reps)
    model = (max(pieces["gather"], pieces["fwd_local"]) + pieces["fwd_dist"] + pieces["bwd_dist"] +
             max(pieces["scatter"], pieces["bwd_local"]))
    out = {"model": args.model, "cp_degree": args.cp, "rank": r, "cut": args.cut, "source": args.source,
           "distributed_seq": args.seq_len, "local_seqs": len(short), "local_tokens": int(sum(short)),
           "exchanged_rows": rb.remote_rows,
           "exchanged_bytes_each_way": int(rb.remote_rows * hk * d * 2 * 2),
           "pieces_ms": pieces, "serial_ms": round(serial, 4), "overlapped_ms": round(overlapped, 4),
           "eq2_model_ms": round(model, 4), "hidden_ms": round(serial - overlapped, 4)}
    rb.destroy()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())

"""How evenly the cost-ordered work lists load the 256 compute units.

The plan sorts the tile work items by descending quadratic cost and the hardware hands
workgroups out in grid order, so the heaviest remaining item always goes to the first
compute unit that frees up: the paper's least-loaded-first rule (Alg. 1, argmin over the
rank loads L; Alg. 2's FLOPs bin-packing) applied to compute units.  This driver measures
what that achieves: with the library's opt-in per-workgroup trace every workgroup of the
forward, dQ and dK/dV kernels records its start and end on the chip-wide 100 MHz counter and
the compute unit it ran on, and per kernel it reports

    span          last end - first start of any workgroup
    busy          mean over the compute units of (time covered by its workgroups) / span
    tail          1 - busy measured from the moment the first compute unit has run dry, i.e.
                  the share of CU-time lost at the end of the launch
    lpt_bound     the same list scheduled greedily (each item to the unit that is free
                  first) with the MEASURED workgroup durations: what ideal dispatch would give

    python -m paper_2505_19609_amd.balance --config 3
"""
from __future__ import annotations

import argparse
import heapq
import json
import sys

import numpy as np

REC = np.dtype([("t0", "<u8"), ("t1", "<u8"), ("hw_id", "<u4"), ("xcc_id", "<u4"), ("block", "<u4"), ("one", "<u4")])
TICK_US = 0.01   # s_memrealtime runs at 100 MHz


def analyse(rec, slots_per_cu):
    """rec: structured records of one launch (written ones only)."""
    t0 = rec["t0"].astype(np.int64)
    t1 = rec["t1"].astype(np.int64)
    start, end = t0.min(), t1.max()
    span = float(end - start)
    # a compute unit: die, shader engine, shader array, CU
    cu = (rec["xcc_id"].astype(np.int64) & 0xF) << 16 | (rec["hw_id"].astype(np.int64) & 0xFF00)
    units = np.unique(cu)
    covered, last_end = [], []
    for u in units:
        sel = np.nonzero(cu == u)[0]
        order = sel[np.argsort(t0[sel])]
        tot, cur_s, cur_e = 0, None, None
        for i in order:               # union of this unit's intervals
            if cur_e is None or t0[i] > cur_e:
                if cur_e is not None:
                    tot += cur_e - cur_s
                cur_s, cur_e = t0[i], t1[i]
            else:
                cur_e = max(cur_e, t1[i])
        tot += cur_e - cur_s
        covered.append(tot)
        last_end.append(t1[sel].max())
    covered, last_end = np.array(covered, float), np.array(last_end, float)
    first_dry = last_end.min()
    tail_lost = float((end - last_end).sum()) / (len(units) * span)
    dur = (t1 - t0).astype(float)
    # greedy list scheduling of the same durations in grid order over the same number of slots
    slots = [0.0] * (len(units) * slots_per_cu)
    heapq.heapify(slots)
    for b in np.argsort(rec["block"]):
        heapq.heappush(slots, heapq.heappop(slots) + dur[b])
    lpt_span = max(slots)
    return {"workgroups": int(len(rec)), "compute_units": int(len(units)),
            "dies": int(len(np.unique(rec["xcc_id"] & 0xF))),
            "span_us": round(span * TICK_US, 2),
            "busy": round(float(covered.mean()) / span, 4),
            "tail_lost": round(tail_lost, 4),
            "first_unit_dry_at": round(float(first_dry - start) / span, 4),
            "wg_us_min_med_max": [round(float(x) * TICK_US, 2) for x in (dur.min(), np.median(dur), dur.max())],
            "sum_wg_time_over_units_x_span": round(float(dur.sum()) / (len(units) * slots_per_cu * span), 4),
            "greedy_span_us": round(lpt_span * TICK_US, 2),
            "span_over_greedy": round(span / lpt_span, 4),
            "ideal_span_us": round(float(dur.sum()) / (len(units) * slots_per_cu) * TICK_US, 2)}


def main(argv=None):
    from . import workloads as W
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--shard-index", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--dump", default=None, help="also write the raw records of the three kernels to this .npz file")
    args = ap.parse_args(argv)
    import torch
    from . import binding as B
    if not torch.cuda.is_available():
        print("balance: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    w = W.config(args.config, args.shard_index) if args.config in (4, 5) else W.config(args.config)
    plan = B.skrull_attn_plan(w.seq_len, w.shard_degree, w.shard_index, w.num_q_heads, w.num_kv_heads,
                              w.head_dim, w.softmax_scale)
    Tq, Tk, Hq, Hkv, d = plan.total_q, plan.total_k, w.num_q_heads, w.num_kv_heads, w.head_dim
    gen = torch.Generator(device="cuda").manual_seed(w.value_seed)
    rnd = lambda rows, h: torch.randn((rows, h, d), generator=gen, device="cuda", dtype=torch.float32).bfloat16()  # noqa: E731
    q, k, v, do = rnd(Tq, Hq), rnd(Tk, Hkv), rnd(Tk, Hkv), rnd(Tq, Hq)
    o, dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    lse = torch.empty((Hq, Tq), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(int(plan.bwd_workspace_bytes), 16), dtype=torch.uint8, device="cuda")
    first, num = B.skrull_attn_trace_layout(plan)
    records = torch.zeros((sum(num), REC.itemsize), dtype=torch.uint8, device="cuda")

    def step():
        B.skrull_attn_fwd(plan, q, k, v, o, lse)
        B.skrull_attn_bwd(plan, q, k, v, o, lse, do, dq, dk, dv, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    B.skrull_attn_trace(records)
    step()
    torch.cuda.synchronize()
    B.skrull_attn_trace(None)
    rec = records.cpu().numpy().view(REC).reshape(-1)
    info = plan.info
    # workgroups of one compute unit at a time: the 8-wavefront forward / dQ shapes and dK/dV fill one alone
    slots = {"fwd": 2 if info.wg_query_rows == 128 else 1,
             "dq": 2 if (info.wg_query_rows == 128 and d == 64) else 1,
             "dkv": 1}
    out = {"workload": w.name, "block_m": int(info.block_m), "block_n": int(info.block_n),
           "head_split": int(info.head_split), "wg_query_rows": int(info.wg_query_rows), "kernels": {}}
    for name, f, n in zip(("fwd", "dq", "dkv"), first, num):
        r = rec[f:f + n]
        r = r[r["one"] == 1]
        out["kernels"][name] = analyse(r, slots[name])
        out["kernels"][name]["grid"] = n
    if args.dump:
        np.savez_compressed(args.dump, **{name: rec[f:f + n] for name, f, n in zip(("fwd", "dq", "dkv"), first, num)})
    plan.destroy()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())

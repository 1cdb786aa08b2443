#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: plan + forward + backward of packed
varlen causal attention over one synthetic micro-batch.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3]

One "step" = skrull_attn_plan + skrull_attn_fwd + skrull_attn_bwd on the
Llama-3-8B-shaped mixed-length micro-batch (config 3; 32,768 tokens: one
24,576-token sequence + short ones).  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line: useful causal TFLOP/s (14*A*d*Hq flops
per step, A = attended pairs), a roofline object for the dominant kernel
(timed live with HIP events on the launch stream) and the CPU oracle timed on
a bounded sample of the same micro-batch.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published


def cpu_baseline(w, np):
    """The fp64 oracle, as it stands, on a bounded sample: the local (short)
    sequences of the micro-batch, all heads, full forward + backward."""
    import oracle
    from paper_2505_19609_amd import workloads as W
    keep = [k for k in range(len(w.seq_len)) if w.shard_degree[k] == 1 and w.seq_len[k] <= 8192]
    # bound the sample to about 1.2e7 attended pairs (10-30 s of CPU work)
    S, pairs = [], 0
    for k in keep:
        L = w.seq_len[k]
        if pairs + L * (L + 1) // 2 > 1.2e7 and S:
            continue
        S.append(L)
        pairs += L * (L + 1) // 2
    desc = oracle.ranges(S)
    sub = W.Workload("sample", S, [1] * len(S), [0] * len(S), w.num_q_heads, w.num_kv_heads,
                     w.head_dim, w.softmax_scale, w.value_seed + 7)
    vals = W.make_values(sub, desc["total_q"], desc["total_k"])
    f = {n: W.bf16_bits_to_f32(a) for n, a in vals.items()}
    t0 = time.perf_counter()
    O, LSE = oracle.attention_fwd(f["q"], f["k"], f["v"], desc, w.softmax_scale)
    dQ, dK, dV, _ = oracle.attention_bwd(f["q"], f["k"], f["v"], f["do"], desc, w.softmax_scale)
    dt = time.perf_counter() - t0
    useful = 14 * oracle.attended_pairs(desc) * w.head_dim * w.num_q_heads
    out = {"value": useful / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(),
           "kind": "oracle", "seconds": round(dt, 3),
           "sample": f"{len(S)} short sequences of the micro-batch ({sum(S)} tokens, "
                     f"{oracle.attended_pairs(desc)} pairs), all {w.num_q_heads} query heads, fp64 fwd+bwd"}
    # the library on the same sample, outside every timed region: largest deviation from the oracle
    # per output, absolute and in spacings of bf16 at the reference value
    import torch
    from paper_2505_19609_amd import binding as B
    plan = B.skrull_attn_plan(S, [1] * len(S), [0] * len(S), w.num_q_heads, w.num_kv_heads, w.head_dim,
                              w.softmax_scale)
    dev = {n: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16) for n, a in vals.items()}
    o, dq = torch.empty_like(dev["q"]), torch.empty_like(dev["q"])
    dk, dv = torch.empty_like(dev["k"]), torch.empty_like(dev["k"])
    lse = torch.empty((w.num_q_heads, plan.total_q), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(int(plan.bwd_workspace_bytes), 16), dtype=torch.uint8, device="cuda")
    B.skrull_attn_fwd(plan, dev["q"], dev["k"], dev["v"], o, lse)
    B.skrull_attn_bwd(plan, dev["q"], dev["k"], dev["v"], o, lse, dev["do"], dq, dk, dv, ws)
    torch.cuda.synchronize()
    plan.destroy()
    par = {}
    for name, got, ref in (("O", o, O), ("LSE", lse, LSE), ("dQ", dq, dQ), ("dK", dk, dK), ("dV", dv, dV)):
        err = np.abs(got.float().cpu().numpy() - ref)
        i = np.unravel_index(np.argmax(err), err.shape)
        spacing = 2.0 ** (np.floor(np.log2(max(abs(ref[i]), 2.0 ** -126))) - 7)
        par[name] = {"max_abs": float(f"{err[i]:.3g}"), "in_bf16_spacings": round(float(err[i] / spacing), 2)}
    out["gpu_vs_oracle_on_sample"] = par
    return out


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` on `workload`, as measured offline with
    rocprofv3's FETCH_SIZE / WRITE_SIZE counters (scaled by a plain copy of known
    size; the summary file gives the commands), or None if no summary is there."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) == 3 and f[0] == "traffic" and f[1] == kernel:
            return int(float(f[2]))
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, help="benchmark micro-batch 1..5 (default 3)")
    ap.add_argument("--shard-index", type=int, default=None)
    ap.add_argument("--block-m", type=int, default=0)
    ap.add_argument("--block-n", type=int, default=0)
    ap.add_argument("--reuse-plan", action="store_true",
                    help="build the plan once instead of in every step (a caller whose micro-batch shape repeats "
                         "can do that; the default, a new plan per step, is what value is quoted on)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--balance", action="store_true",
                    help="with --config 4: also time the same micro-batch with the first slice instead of the last "
                         "(or the other way round) and print the time ratio beside the pair ratio")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (a kernel of known traffic, "
                         "to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters against)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding across "
              "GPUs); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2505_19609_amd import binding as B
    from paper_2505_19609_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    w = W.config(args.config, args.shard_index) if args.config in (4, 5) else W.config(args.config)

    def run_workload(w, steps, warmup, copy_probe=False):
        """Time `steps` steps (plan + forward + backward) of micro-batch `w`; tensors resident in HBM."""
        def make_plan():
            return B.skrull_attn_plan(w.seq_len, w.shard_degree, w.shard_index, w.num_q_heads,
                                      w.num_kv_heads, w.head_dim, w.softmax_scale, args.block_m,
                                      args.block_n)

        plan = make_plan()
        Tq, Tk, Hq, Hkv, d = plan.total_q, plan.total_k, w.num_q_heads, w.num_kv_heads, w.head_dim
        # synthetic N(0,1) bf16 tensors drawn on the device (values do not affect cost)
        gen = torch.Generator(device="cuda").manual_seed(w.value_seed)
        q = torch.randn((Tq, Hq, d), generator=gen, device="cuda", dtype=torch.float32).mul_(w.q_prescale).bfloat16()
        k = torch.randn((Tk, Hkv, d), generator=gen, device="cuda", dtype=torch.float32).bfloat16()
        v = torch.randn((Tk, Hkv, d), generator=gen, device="cuda", dtype=torch.float32).bfloat16()
        do = torch.randn((Tq, Hq, d), generator=gen, device="cuda", dtype=torch.float32).bfloat16()
        o, dq = torch.empty_like(q), torch.empty_like(q)
        dk, dv = torch.empty_like(k), torch.empty_like(v)
        lse = torch.empty((Hq, Tq), dtype=torch.float32, device="cuda")
        ws = torch.empty(max(int(plan.bwd_workspace_bytes), 16), dtype=torch.uint8, device="cuda")
        info = plan.info
        r = {"pairs": int(plan.attended_pairs), "useful": int(plan.useful_flops_fwd + plan.useful_flops_bwd),
             "Tq": Tq, "Tk": Tk,
             # what the plan has in effect (block_n, head_split and the workgroup shape are the
             # library's choice unless given)
             "shape": {"block_m": int(info.block_m), "block_n": int(info.block_n),
                       "fwd_items": int(info.n_fwd_items), "dkv_items": int(info.n_dkv_items),
                       "wg_query_rows": int(info.wg_query_rows), "head_split": int(info.head_split)}}
        plan.destroy()
        for _ in range(warmup):
            p = make_plan()
            B.skrull_attn_fwd(p, q, k, v, o, lse)
            B.skrull_attn_bwd(p, q, k, v, o, lse, do, dq, dk, dv, ws)
            p.destroy()
        torch.cuda.synchronize()
        if copy_probe:
            src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
            dst = torch.empty_like(src)
            dst.copy_(src)  # reads 1 GiB, writes 1 GiB
            torch.cuda.synchronize()
            del src, dst
        B.skrull_attn_profile(True)
        kms = np.zeros((steps, 4))
        t_plan = np.zeros(steps)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        kept = make_plan() if args.reuse_plan else None
        for i in range(steps):
            tp = time.perf_counter()
            p = kept or make_plan()
            t_plan[i] = time.perf_counter() - tp
            B.skrull_attn_fwd(p, q, k, v, o, lse)
            B.skrull_attn_bwd(p, q, k, v, o, lse, do, dq, dk, dv, ws)
            kms[i] = B.skrull_attn_profile_read()  # waits for this step's kernels
            if kept is None:
                p.destroy()
        torch.cuda.synchronize()
        r["wall_s"] = time.perf_counter() - t0
        if kept is not None:
            kept.destroy()
        B.skrull_attn_profile(False)
        r["kms"], r["t_plan"] = kms, t_plan
        return r

    r = run_workload(w, args.steps, args.warmup, args.copy_probe)
    Hq, Hkv, d = w.num_q_heads, w.num_kv_heads, w.head_dim
    pairs, useful, Tq, Tk = r["pairs"], r["useful"], r["Tq"], r["Tk"]
    kms_all = r["kms"]
    kms = kms_all.mean(axis=0)
    ms_step = r["wall_s"] / args.steps * 1e3
    tflops = useful / (r["wall_s"] / args.steps) / 1e12
    # the same step from the kernels' own HIP events (forward + dQ + dK/dV), median over the steps:
    # what is left of the wall clock is the plan (built every step, reported on its own), the
    # synchronisation it needs and the read-back of the events
    ev_step = np.median(kms_all[:, 0] + kms_all[:, 2] + kms_all[:, 3])
    ev_min = np.min(kms_all[:, 0] + kms_all[:, 2] + kms_all[:, 3])

    # dominant kernel and its algorithmic flops per launch:
    #   forward 4*A*d*Hq; dK/dV kernel 8*A*d*Hq (S, dP, dV, dK); dQ kernel 2*A*d*Hq
    #   (its recomputation of S and dP is not algorithmic work)
    unit = pairs * d * Hq
    kernels = {"fwd_kernel": (kms[0], 4 * unit), "dkv_kernel": (kms[2], 8 * unit), "dq_kernel": (kms[3], 2 * unit)}
    dom = max(kernels, key=lambda n: kernels[n][0])
    ach = kernels[dom][1] / (kernels[dom][0] * 1e-3) / 1e12
    # the matrix-pipe rate this GPU actually sustains (clock under load), beside the nominal peak
    ceiling = B.skrull_attn_mfma_ceiling()
    # HBM bytes per launch measured offline (rocprofv3 FETCH_SIZE / WRITE_SIZE; the file gives the commands)
    traffic = {n: measured_traffic(w.name, n) for n in kernels}
    have_traffic = all(v is not None for v in traffic.values())
    # algorithmic bytes of a step (bf16 tensors read / written once, fp32 LSE and the D workspace)
    alg_bytes = (12 * d * Hq + 4 * Hq + 12 * Hq) * Tq + 12 * d * Hkv * Tk
    roofline = {"bound": "mfma", "kernel": dom, "achieved": round(ach, 2), "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": round(ach / PEAK_BF16_TFLOPS, 4),
                "traffic": traffic[dom], "traffic_source": "offline rocprofv3 counters, profiles/hbm_traffic_%s.txt" % w.name
                if traffic[dom] is not None else None,
                "mfma_only_measured": round(ceiling, 1), "frac_of_measured": round(ach / ceiling, 4),
                "kernel_ms": {"fwd": round(float(kms[0]), 4), "dkv": round(float(kms[2]), 4),
                              "dq": round(float(kms[3]), 4)},
                "kernel_tflops": {n.split("_")[0]: round(f / (t * 1e-3) / 1e12, 1) for n, (t, f) in kernels.items()},
                # what the kernels execute on unmasked pairs: the dQ kernel recomputes S and dP (6 instead of 2
                # flops per pair, head and head dim), the other two execute what they are credited with
                "kernel_executed_tflops": {"fwd": round(4 * unit / (kms[0] * 1e-3) / 1e12, 1),
                                           "dkv": round(8 * unit / (kms[2] * 1e-3) / 1e12, 1),
                                           "dq": round(6 * unit / (kms[3] * 1e-3) / 1e12, 1),
                                           "step": round(18 * unit / (ev_step * 1e-3) / 1e12, 1),
                                           "step_frac_of_mfma_only_measured": round(18 * unit / (ev_step * 1e-3) / 1e12 / ceiling, 4)},
                "hbm": {"algorithmic_bytes_per_step": int(alg_bytes),
                        "algorithmic_gbps": round(alg_bytes / (ev_step * 1e-3) / 1e9, 1),
                        "measured_bytes_per_step": int(sum(traffic.values())) if have_traffic else None,
                        "measured_gbps": round(sum(traffic.values()) / (ev_step * 1e-3) / 1e9, 1) if have_traffic else None,
                        "peak_gbps": 8000.0}}
    out = {
        "metric": "varlen causal attn fwd+bwd useful TFLOP/s, 1 GPU",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "frac_of_bf16_mfma_peak": round(tflops / PEAK_BF16_TFLOPS, 4),
        "tflops_fwd": round(4 * unit / (kms[0] * 1e-3) / 1e12, 2),
        "tflops_bwd": round(10 * unit / ((kms[2] + kms[3]) * 1e-3) / 1e12, 2),
        "kernels_only": {"ms_median": round(float(ev_step), 4), "ms_min": round(float(ev_min), 4),
                         "tflops": round(useful / (ev_step * 1e-3) / 1e12, 2),
                         "note": "fwd + dQ + dK/dV from HIP events on the launch stream, median over the steps; "
                                 "value above is the wall clock of plan + fwd + bwd"},
        "config": {"workload": w.name, "num_seqs": len(w.seq_len), "total_q": Tq, "total_k": Tk,
                   "q_heads": Hq, "kv_heads": Hkv, "head_dim": d, "attended_pairs": pairs,
                   "useful_flops_per_step": useful, **r["shape"],
                   "step": "fwd + bwd (plan reused)" if args.reuse_plan else "plan + fwd + bwd", "ms_plan": round(float(np.median(r["t_plan"])) * 1e3, 4)},
        "roofline": roofline,
    }
    if args.config == 4 and args.balance:
        # Eq. 4 charges every rank of a distributed sequence FLOPs/N; under the causal mask the
        # contiguous slice r attends (2r+1)/N^2 of the pairs.  The same micro-batch with the first
        # slice instead of the last, side by side.
        other = 0 if w.shard_index[0] != 0 else w.shard_degree[0] - 1
        w2 = W.config(4, other)
        r2 = run_workload(w2, max(3, args.steps // 2), 2)
        ev2 = float(np.median(r2["kms"][:, 0] + r2["kms"][:, 2] + r2["kms"][:, 3]))
        out["shard_balance"] = {"index": int(w.shard_index[0]), "other_index": int(other),
                                "ms": round(float(ev_step), 4), "other_ms": round(ev2, 4),
                                "time_ratio": round(float(ev_step) / ev2, 3),
                                "pair_ratio": round(pairs / r2["pairs"], 3),
                                "other_tflops": round(r2["useful"] / (ev2 * 1e-3) / 1e12, 2)}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, np)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

"""Helpers for the GPU parity tests: run the HIP library through its binding
and fetch results as numpy arrays.  No method arithmetic here."""
import numpy as np


def to_dev(bits):
    import torch
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def run_library(w, block_m=0, block_n=0, vals=None, backward=True, keep_device=False, head_split=0,
                wg_query_rows=0):
    """Plan + forward (+ backward) of workload ``w`` on the current GPU."""
    import torch
    from paper_2505_19609_amd import binding as B
    from paper_2505_19609_amd import workloads as W

    plan = B.skrull_attn_plan(w.seq_len, w.shard_degree, w.shard_index, w.num_q_heads,
                              w.num_kv_heads, w.head_dim, w.softmax_scale, block_m, block_n,
                              shard_cut=w.shard_cut, head_split=head_split, wg_query_rows=wg_query_rows)
    if vals is None:
        vals = W.make_values(w, plan.total_q, plan.total_k)
    dev = {n: to_dev(a) for n, a in vals.items()}
    o = torch.full_like(dev["q"], float("nan"))
    lse = torch.full((w.num_q_heads, plan.total_q), float("nan"), dtype=torch.float32, device="cuda")
    B.skrull_attn_fwd(plan, dev["q"], dev["k"], dev["v"], o, lse)
    out = {"plan": plan, "vals": vals}
    if backward:
        dq = torch.full_like(dev["q"], float("nan"))
        dk = torch.full_like(dev["k"], float("nan"))
        dv = torch.full_like(dev["v"], float("nan"))
        ws = torch.empty(max(int(plan.bwd_workspace_bytes), 16), dtype=torch.uint8, device="cuda")
        B.skrull_attn_bwd(plan, dev["q"], dev["k"], dev["v"], o, lse, dev["do"], dq, dk, dv, ws)
    torch.cuda.synchronize()
    res = {"o": o, "lse": lse}
    if backward:
        res.update(dq=dq, dk=dk, dv=dv)
    if keep_device:
        out["dev"] = res
        out["dev_in"] = dev
    for n, t in res.items():
        out[n] = t.float().cpu().numpy()
    return out


def widen(vals):
    from paper_2505_19609_amd import workloads as W
    return {n: W.bf16_bits_to_f32(a) for n, a in vals.items()}


def bf16_ulp(x):
    """Spacing of bf16 numbers around |x| (8 significand bits)."""
    ax = np.maximum(np.abs(x), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(ax)) - 7)

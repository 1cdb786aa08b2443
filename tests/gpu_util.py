"""Helpers for the GPU parity tests: run the HIP library through its binding
and fetch results as numpy arrays.  No method arithmetic here."""
import numpy as np


def to_dev(bits):
    import torch
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


GUARD = 2048        # elements of margin on each side of a guarded tensor (a multiple of 16 bytes)
GUARD_VALUE = 12352.0  # exact in bf16 and fp32; no kernel output of the tests comes near it


def guarded(shape, dtype, fill):
    """A tensor of `shape` filled with `fill`, inside a larger buffer whose margins hold GUARD_VALUE
    (uint8: 0xA5).  Returns (whole buffer, the tensor)."""
    import torch
    n = int(np.prod(shape))
    mark = 0xA5 if dtype == torch.uint8 else GUARD_VALUE
    buf = torch.full((n + 2 * GUARD,), mark, dtype=dtype, device="cuda")
    view = buf[GUARD:GUARD + n]
    view.fill_(fill)
    return buf, view.view(shape)


def margins_intact(buf):
    import torch
    mark = 0xA5 if buf.dtype == torch.uint8 else GUARD_VALUE
    return bool((buf[:GUARD] == mark).all().item()) and bool((buf[-GUARD:] == mark).all().item())


def run_library(w, block_m=0, block_n=0, vals=None, backward=True, keep_device=False, head_split=0,
                wg_query_rows=0, guard=False):
    """Plan + forward (+ backward) of workload ``w`` on the current GPU.  With `guard` every
    output and the workspace sit between margins that are checked afterwards: out["margins"]
    names the tensors whose margins were written to (none, if every store stayed inside)."""
    import torch
    from paper_2505_19609_amd import binding as B
    from paper_2505_19609_amd import workloads as W

    plan = B.skrull_attn_plan(w.seq_len, w.shard_degree, w.shard_index, w.num_q_heads,
                              w.num_kv_heads, w.head_dim, w.softmax_scale, block_m, block_n,
                              shard_cut=w.shard_cut, head_split=head_split, wg_query_rows=wg_query_rows)
    if vals is None:
        vals = W.make_values(w, plan.total_q, plan.total_k)
    dev = {n: to_dev(a) for n, a in vals.items()}
    bufs = {}

    def alloc(name, shape, dtype, fill=float("nan")):
        if not guard:
            return torch.full(shape, fill, dtype=dtype, device="cuda")
        bufs[name], t = guarded(shape, dtype, fill)
        return t

    o = alloc("o", tuple(dev["q"].shape), torch.bfloat16)
    lse = alloc("lse", (w.num_q_heads, plan.total_q), torch.float32)
    B.skrull_attn_fwd(plan, dev["q"], dev["k"], dev["v"], o, lse)
    out = {"plan": plan, "vals": vals}
    if backward:
        dq = alloc("dq", tuple(dev["q"].shape), torch.bfloat16)
        dk = alloc("dk", tuple(dev["k"].shape), torch.bfloat16)
        dv = alloc("dv", tuple(dev["v"].shape), torch.bfloat16)
        ws = alloc("workspace", (max(int(plan.bwd_workspace_bytes), 16),), torch.uint8, 0)
        B.skrull_attn_bwd(plan, dev["q"], dev["k"], dev["v"], o, lse, dev["do"], dq, dk, dv, ws)
    torch.cuda.synchronize()
    if guard:
        out["margins"] = [n for n, b in bufs.items() if not margins_intact(b)]
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

"""torch.autograd wrapper around the library's forward / backward, for callers that
train with PyTorch: argument marshalling and bookkeeping only, every step of the
attention runs in the HIP kernels behind the C ABI."""
from __future__ import annotations

import torch

from . import binding as B


class _SkrullAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, plan):
        if not (q.is_cuda and q.dtype == torch.bfloat16 and q.is_contiguous() and k.is_contiguous()
                and v.is_contiguous() and k.dtype == torch.bfloat16 and v.dtype == torch.bfloat16):
            raise ValueError("q, k, v must be contiguous bf16 CUDA tensors")
        if q.shape != (plan.total_q, plan.num_q_heads, plan.head_dim) or \
                k.shape != (plan.total_k, plan.num_kv_heads, plan.head_dim) or v.shape != k.shape:
            raise ValueError("tensor shapes do not match the plan")
        o = torch.empty_like(q)
        lse = torch.empty((plan.num_q_heads, plan.total_q), dtype=torch.float32, device=q.device)
        B.skrull_attn_fwd(plan, q, k, v, o, lse)
        ctx.plan = plan
        ctx.save_for_backward(q, k, v, o, lse)
        return o

    @staticmethod
    def backward(ctx, d_o):
        q, k, v, o, lse = ctx.saved_tensors
        plan = ctx.plan
        d_o = d_o.contiguous()
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        ws = torch.empty(max(int(plan.bwd_workspace_bytes), 16), dtype=torch.uint8, device=q.device)
        B.skrull_attn_bwd(plan, q, k, v, o, lse, d_o, dq, dk, dv, ws)
        return dq, dk, dv, None


def skrull_attention(q, k, v, plan):
    """O = packed varlen causal attention of the micro-batch `plan` describes
    (a binding.Plan); differentiable with respect to q, k, v."""
    return _SkrullAttention.apply(q, k, v, plan)

"""skrull_attn_bwd_static, the backward entry point that allocates nothing (its workspace is a
static device array inside the library), through the C ABI against skrull_attn_bwd: the same
kernels on another workspace, so every output must be the same bits.  Two calls in a row, the
second on a smaller micro-batch (the array keeps the first call's contents); a plan whose
workspace exceeds the array is rejected with a message that names both sizes."""
import numpy as np
import pytest

from paper_2505_19609_amd import workloads as W
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


def _both(w, head_split=0):
    import torch
    from paper_2505_19609_amd import binding as B
    plan = B.skrull_attn_plan(w.seq_len, w.shard_degree, w.shard_index, w.num_q_heads, w.num_kv_heads,
                              w.head_dim, w.softmax_scale, shard_cut=w.shard_cut, head_split=head_split)
    vals = W.make_values(w, plan.total_q, plan.total_k)
    dev = {n: to_dev(a) for n, a in vals.items()}
    o = torch.empty_like(dev["q"])
    lse = torch.empty((w.num_q_heads, plan.total_q), dtype=torch.float32, device="cuda")
    B.skrull_attn_fwd(plan, dev["q"], dev["k"], dev["v"], o, lse)
    res = {}
    for which in ("workspace", "static"):
        dq = torch.full_like(dev["q"], float("nan"))
        dk = torch.full_like(dev["k"], float("nan"))
        dv = torch.full_like(dev["v"], float("nan"))
        if which == "workspace":
            ws = torch.empty(max(int(plan.bwd_workspace_bytes), 16), dtype=torch.uint8, device="cuda")
            B.skrull_attn_bwd(plan, dev["q"], dev["k"], dev["v"], o, lse, dev["do"], dq, dk, dv, ws)
        else:
            torch.cuda.synchronize()
            before = torch.cuda.memory_allocated()
            B.skrull_attn_bwd_static(plan, dev["q"], dev["k"], dev["v"], o, lse, dev["do"], dq, dk, dv)
            assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        res[which] = (dq, dk, dv)
    for a, b, n in zip(res["workspace"], res["static"], ("dq", "dk", "dv")):
        assert torch.isfinite(a.float()).all(), n
        assert torch.equal(a.view(torch.int16), b.view(torch.int16)), n
    info = (int(plan.total_q), int(plan.info.head_split))
    plan.destroy()
    return info


def test_static_workspace_gives_the_same_bits_on_two_calls_in_a_row():
    big = W.Workload("static_big", [3000, 700, 129, 2100, 64], [1, 1, 1, 3, 1], [0, 0, 0, 1, 0], 8, 2, 128,
                     128 ** -0.5, 31, shard_cut=[0, 0, 0, 1, 0])
    small = W.Workload("static_small", [300, 65, 1], [1, 1, 1], [0, 0, 0], 8, 2, 128, 128 ** -0.5, 32)
    rows_big, _ = _both(big, head_split=1)
    rows_small, hs = _both(small)       # smaller input on the array the first call left behind
    assert rows_small < rows_big and hs > 1   # (its few work items make the plan split the heads)
    # with the fp32 partial sums of a head split in the array as well, then again without
    w = W.Workload("static_split", [1024, 300], [1, 1], [0, 0], 14, 2, 64, 0.125, 33)
    _, hs = _both(w, head_split=7)
    assert hs == 7
    _both(small)


def test_static_workspace_rejects_what_does_not_fit():
    from paper_2505_19609_amd import binding as B
    import torch
    # 14 query heads x 40,000 rows x 8 bytes = 4.5 MB, plus 2 x 7 shares x 40,000 x 2 x 64 x 4 = 287 MB
    plan = B.skrull_attn_plan([40000], [1], [0], 14, 2, 64, 0.125, head_split=7)
    assert plan.bwd_workspace_bytes > B.STATIC_SCRATCH_BYTES
    t = torch.zeros(64, dtype=torch.bfloat16, device="cuda")   # never read: the call fails first
    with pytest.raises(B.SkrullError) as e:
        B.skrull_attn_bwd_static(plan, t, t, t, t, t.float(), t, t, t, t)
    assert e.value.code == B.SKRULL_EINVAL and str(B.STATIC_SCRATCH_BYTES) in str(e.value)
    plan.destroy()
    # the same micro-batch without the split fits
    plan = B.skrull_attn_plan([40000], [1], [0], 14, 2, 64, 0.125, head_split=1)
    assert plan.bwd_workspace_bytes <= B.STATIC_SCRATCH_BYTES
    plan.destroy()


def test_null_arguments_of_the_static_entry_point():
    from paper_2505_19609_amd import binding as B
    assert B.lib().skrull_attn_bwd_static(*([None] * 11)) == B.SKRULL_EINVAL

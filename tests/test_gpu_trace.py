"""The opt-in per-workgroup trace (a measurement aid): every workgroup that has work writes one
record, results do not change, and a buffer that is too small is refused."""
import numpy as np
import pytest

from paper_2505_19609_amd import workloads as W
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("d", [64, 128])
def test_trace_records_every_workgroup_and_changes_nothing(d):
    import torch
    from paper_2505_19609_amd import binding as B
    from paper_2505_19609_amd.balance import REC, analyse
    w = W.Workload("trace", [3000, 129, 700, 2100], [1, 1, 1, 3], [0, 0, 0, 1], 8, 2, d, d ** -0.5, 17)
    plan = B.skrull_attn_plan(w.seq_len, w.shard_degree, w.shard_index, 8, 2, d, w.softmax_scale)
    vals = W.make_values(w, plan.total_q, plan.total_k)
    dev = {n: to_dev(a) for n, a in vals.items()}
    first, num = B.skrull_attn_trace_layout(plan)
    assert first == [0, num[0], num[0] + num[1]] and all(n > 0 for n in num)
    outs = []
    for traced in (False, True):
        o, dq = torch.empty_like(dev["q"]), torch.empty_like(dev["q"])
        dk, dv = torch.empty_like(dev["k"]), torch.empty_like(dev["k"])
        lse = torch.empty((8, plan.total_q), dtype=torch.float32, device="cuda")
        ws = torch.empty(max(int(plan.bwd_workspace_bytes), 16), dtype=torch.uint8, device="cuda")
        records = torch.zeros((sum(num), REC.itemsize), dtype=torch.uint8, device="cuda")
        if traced:
            with pytest.raises(B.SkrullError):          # room for the forward only: the backward is refused
                B.skrull_attn_trace(records[:num[0]])
                B.skrull_attn_bwd(plan, dev["q"], dev["k"], dev["v"], o, lse, dev["do"], dq, dk, dv, ws)
            B.skrull_attn_trace(records)
        B.skrull_attn_fwd(plan, dev["q"], dev["k"], dev["v"], o, lse)
        B.skrull_attn_bwd(plan, dev["q"], dev["k"], dev["v"], o, lse, dev["do"], dq, dk, dv, ws)
        torch.cuda.synchronize()
        B.skrull_attn_trace(None)
        outs.append((o, lse, dq, dk, dv))
        if traced:
            rec = records.cpu().numpy().view(REC).reshape(-1)
            for f, n in zip(first, num):
                r = rec[f:f + n]
                r = r[r["one"] == 1]
                assert 0 < len(r) <= n
                assert (r["t1"] >= r["t0"]).all() and (r["t0"] > 0).all()
                assert len(np.unique(r["block"])) == len(r) and r["block"].max() < n
                a = analyse(r, 1)
                assert 0 < a["compute_units"] <= 256 and 0 < a["busy"] <= 1.0
        else:
            assert not records.any()
    for x, y in zip(*outs):
        assert torch.equal(x.view(torch.int16) if x.dtype == torch.bfloat16 else x,
                           y.view(torch.int16) if y.dtype == torch.bfloat16 else y)
    plan.destroy()


def test_profiling_switch_belongs_to_the_calling_thread():
    """One thread profiles, another does not: the second reads nothing back (SKRULL_EINVAL)
    and its calls record no events."""
    import threading
    import torch
    from paper_2505_19609_amd import binding as B
    w = W.config(1)
    plan = B.skrull_attn_plan(w.seq_len, w.shard_degree, w.shard_index, 4, 4, 64, 1.0)
    vals = W.make_values(w, plan.total_q, plan.total_k)
    dev = {n: to_dev(a) for n, a in vals.items()}
    o = torch.empty_like(dev["q"])
    lse = torch.empty((4, plan.total_q), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    B.skrull_attn_profile(True)
    B.skrull_attn_fwd(plan, dev["q"], dev["k"], dev["v"], o, lse, stream=stream)
    seen = {}

    def other():
        torch.cuda.set_device(0)
        try:
            B.skrull_attn_profile_read()
        except B.SkrullError as e:
            seen["code"] = e.code
        B.skrull_attn_fwd(plan, dev["q"], dev["k"], dev["v"], o, lse, stream=stream)

    t = threading.Thread(target=other)
    t.start(); t.join()
    ms = B.skrull_attn_profile_read()
    B.skrull_attn_profile(False)
    torch.cuda.synchronize()
    assert seen.get("code") == B.SKRULL_EINVAL
    assert ms[0] > 0 and ms[2] == -1 and ms[3] == -1
    with pytest.raises(B.SkrullError):
        B.skrull_attn_profile_read()          # switched off again
    plan.destroy()

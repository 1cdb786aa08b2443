"""The forward and backward entry points only enqueue kernels on the caller's stream
(no allocation, no memset, no synchronisation), so a launch-bound inner loop can be
captured in a HIP graph.  Capture one forward + backward, replay it several times with
eager work and synchronisations in between, and compare every replay bit for bit with
the eager result on the same inputs."""
import numpy as np
import pytest
import torch

from paper_2505_19609_amd import workloads as W
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


SMALL = ([700, 129, 2100, 64], [1, 1, 3, 1], [0, 0, 1, 0], [0, 0, 1, 0])
# more work items than the chip holds workgroups at once: the persistent launches with their
# work queues (and the kernels that clear them) are what is captured
LARGE = ([9000, 700, 6100, 64], [1, 1, 3, 1], [0, 0, 1, 0], [0, 0, 1, 0])


@pytest.mark.parametrize("heads,d,split,lengths", [((4, 2), 64, 0, SMALL), ((14, 2), 64, 3, SMALL), ((8, 2), 128, 1, SMALL),
                                                   ((16, 4), 128, 1, LARGE), ((14, 2), 64, 0, LARGE)])
def test_graph_replays_equal_eager(heads, d, split, lengths):
    from paper_2505_19609_amd import binding as B
    w = W.Workload("graph", lengths[0], lengths[1], lengths[2], heads[0], heads[1], d,
                   d ** -0.5, 4321, shard_cut=lengths[3])
    plan = B.skrull_attn_plan(w.seq_len, w.shard_degree, w.shard_index, heads[0], heads[1], d,
                              w.softmax_scale, shard_cut=w.shard_cut, head_split=split)
    vals = W.make_values(w, plan.total_q, plan.total_k)
    dev = {n: to_dev(a) for n, a in vals.items()}
    outs = {n: torch.empty_like(dev[src]) for n, src in (("o", "q"), ("dq", "q"), ("dk", "k"), ("dv", "k"))}
    lse = torch.empty((heads[0], plan.total_q), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(int(plan.bwd_workspace_bytes), 16), dtype=torch.uint8, device="cuda")

    def step():
        B.skrull_attn_fwd(plan, dev["q"], dev["k"], dev["v"], outs["o"], lse)
        B.skrull_attn_bwd(plan, dev["q"], dev["k"], dev["v"], outs["o"], lse, dev["do"],
                          outs["dq"], outs["dk"], outs["dv"], ws)

    step()
    torch.cuda.synchronize()
    eager = {n: t.clone() for n, t in outs.items()}
    eager["lse"] = lse.clone()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):   # warm-up on the capture stream
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for rep in range(4):
        for t in list(outs.values()) + [lse, ws]:
            t.view(torch.uint8).fill_(0xFF if rep % 2 else 0)   # the program's own eager work in between
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n, t in outs.items():
            assert torch.equal(t, eager[n]), (rep, n)
        assert torch.equal(lse, eager["lse"]), rep
    plan.destroy()


def test_forward_calls_of_one_plan_overlap_on_two_streams():
    """A plan's forward calls take the plan's work-queue slots in turn, so calls that overlap on
    different streams do not share a queue: two streams run the same plan's forward at the same
    time, several times over, and every output equals the one-stream result bit for bit."""
    from paper_2505_19609_amd import binding as B
    heads, d = (16, 4), 128
    w = W.Workload("two_streams", [9000, 700, 4000], [1, 1, 1], [0, 0, 0], heads[0], heads[1], d, d ** -0.5, 99)
    plan = B.skrull_attn_plan(w.seq_len, w.shard_degree, w.shard_index, heads[0], heads[1], d, w.softmax_scale)
    first, num = B.skrull_attn_trace_layout(plan)
    assert num[0] > 256          # more work items than compute units: the launch is persistent
    vals = W.make_values(w, plan.total_q, plan.total_k)
    dev = {n: to_dev(a) for n, a in vals.items()}
    ref_o = torch.empty_like(dev["q"])
    ref_lse = torch.empty((heads[0], plan.total_q), dtype=torch.float32, device="cuda")
    B.skrull_attn_fwd(plan, dev["q"], dev["k"], dev["v"], ref_o, ref_lse)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = [(torch.empty_like(ref_o), torch.empty_like(ref_lse)) for _ in streams]
    for rep in range(40):        # wraps around the plan's 64 slots
        for st, (o, lse) in zip(streams, outs):
            if rep % 8 == 0:
                o.fill_(float("nan")); lse.fill_(float("nan"))
            st.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(st):
                B.skrull_attn_fwd(plan, dev["q"], dev["k"], dev["v"], o, lse)
        if rep % 8 == 7:
            torch.cuda.synchronize()
            for o, lse in outs:
                assert torch.equal(o.view(torch.int16), ref_o.view(torch.int16)), rep
                assert torch.equal(lse, ref_lse), rep
    torch.cuda.synchronize()
    plan.destroy()

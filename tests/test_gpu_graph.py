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


@pytest.mark.parametrize("heads,d,split", [((4, 2), 64, 0), ((14, 2), 64, 3), ((8, 2), 128, 1)])
def test_graph_replays_equal_eager(heads, d, split):
    from paper_2505_19609_amd import binding as B
    w = W.Workload("graph", [700, 129, 2100, 64], [1, 1, 3, 1], [0, 0, 1, 0], heads[0], heads[1], d,
                   d ** -0.5, 4321, shard_cut=[0, 0, 1, 0])
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

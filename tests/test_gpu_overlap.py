"""The two-stream order (gather of the distributed sequences' K/V hidden behind the local
sequences' forward, their dK/dV leaving behind the local sequences' backward; Eq. 2)
against the plain one-stream order and against one plan over the whole micro-batch:
every output bit for bit; and the overlapped order's outputs against the fp64 oracle of the
same micro-batch at the stated tolerances."""
import json

import numpy as np
import pytest
import torch

from paper_2505_19609_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("source", ["host", "device"])
@pytest.mark.parametrize("cut", [0, 1])
def test_overlapped_order_changes_no_bit(oracle, source, cut):
    from paper_2505_19609_amd import binding as B
    from paper_2505_19609_amd.overlap_run import RankBatch

    heads, d = (4, 2), 64
    loc = ([300, 64, 777], [1, 1, 1], [0, 0, 0], [0, 0, 0])
    dist = ([4096, 1001], [4, 4], [3, 1], [cut, cut])
    rb = RankBatch(loc, dist, heads, d, 5, source, head_split=1)   # as the one-plan run below

    def poison():
        for t in rb.parts.values():
            for n in ("o", "lse", "dq", "dk", "dv"):
                t[n].fill_(float("nan"))
        for n in ("dk", "dv"):
            rb.stage[n].fill_(float("nan"))
        dd = rb.parts["dist"]
        dd["k"][:rb.remote_rows].zero_()       # the gather must bring these back
        dd["v"][:rb.remote_rows].zero_()
        torch.cuda.synchronize()

    poison()
    rb.step_serial()
    torch.cuda.synchronize()
    a = rb.outputs()
    for rep in range(3):
        poison()
        rb.step_overlapped()
        torch.cuda.synchronize()
        b = rb.outputs()
        assert a.keys() == b.keys()
        for n in a:
            assert torch.isfinite(a[n].float()).all(), n
            assert torch.equal(a[n], b[n]), (rep, n)
    # what left for the other ranks is the partial gradient of the rows they own
    assert torch.equal(a["stage.dk"].cuda(), a["dist.dk"][:rb.remote_rows])

    # one plan over the whole micro-batch (local first, then distributed): same bits
    L, D = rb.parts["loc"], rb.parts["dist"]
    plan = B.skrull_attn_plan(loc[0] + dist[0], loc[1] + dist[1], loc[2] + dist[2], heads[0], heads[1], d,
                              d ** -0.5, shard_cut=loc[3] + dist[3], head_split=1)
    cat = {n: torch.cat([L[n], D[n]]) for n in ("q", "k", "v", "do")}
    o, dq = torch.empty_like(cat["q"]), torch.empty_like(cat["q"])
    dk, dv = torch.empty_like(cat["k"]), torch.empty_like(cat["k"])
    lse = torch.empty((heads[0], plan.total_q), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(int(plan.bwd_workspace_bytes), 16), dtype=torch.uint8, device="cuda")
    B.skrull_attn_fwd(plan, cat["q"], cat["k"], cat["v"], o, lse)
    B.skrull_attn_bwd(plan, cat["q"], cat["k"], cat["v"], o, lse, cat["do"], dq, dk, dv, ws)
    torch.cuda.synchronize()
    assert torch.equal(o, torch.cat([a["loc.o"], a["dist.o"]]))
    assert torch.equal(lse, torch.cat([a["loc.lse"], a["dist.lse"]], dim=1))
    assert torch.equal(dq, torch.cat([a["loc.dq"], a["dist.dq"]]))
    assert torch.equal(dk, torch.cat([a["loc.dk"], a["dist.dk"]]))
    assert torch.equal(dv, torch.cat([a["loc.dv"], a["dist.dv"]]))
    plan.destroy()

    # the overlapped order against the fp64 oracle (Eq. 2 reorders the pieces of the rank's
    # micro-batch, it must not change what is computed): local sequences, then the slices
    bits = {n: cat[n].view(torch.int16).cpu().numpy().view(np.uint16) for n in cat}
    f = {n: W.bf16_bits_to_f32(a) for n, a in bits.items()}
    desc = oracle.ranges(loc[0] + dist[0], loc[1] + dist[1], loc[2] + dist[2], loc[3] + dist[3])
    O, LSE = oracle.attention_fwd(f["q"], f["k"], f["v"], desc, d ** -0.5)
    dQ, dK, dV, _ = oracle.attention_bwd(f["q"], f["k"], f["v"], f["do"], desc, d ** -0.5)
    got = {"o": torch.cat([b["loc.o"], b["dist.o"]]), "lse": torch.cat([b["loc.lse"], b["dist.lse"]], dim=1),
           "dq": torch.cat([b["loc.dq"], b["dist.dq"]]), "dk": torch.cat([b["loc.dk"], b["dist.dk"]]),
           "dv": torch.cat([b["loc.dv"], b["dist.dv"]])}
    for n, ref, tol in (("o", O, 2e-2), ("lse", LSE, 2e-2), ("dq", dQ, 5e-2), ("dk", dK, 5e-2), ("dv", dV, 5e-2)):
        err = float(np.abs(got[n].float().cpu().numpy() - ref).max())
        print(f"overlapped ({source}, cut {cut}) {n}: max-abs {err:.4g} vs fp64 oracle (tol {tol})")
        assert err <= tol, (n, err)
    # the partial dK/dV rows that left through the staging buffer, against the oracle's
    first_dist_row = int(desc["cu_k"][len(loc[0])])
    for n, ref in (("stage.dk", dK), ("stage.dv", dV)):
        err = float(np.abs(b[n].float().cpu().numpy() - ref[first_dist_row:first_dist_row + rb.remote_rows]).max())
        assert err <= 5e-2, (n, err)
    rb.destroy()


def test_overlap_driver(capsys):
    from paper_2505_19609_amd import overlap_run
    rc = overlap_run.main(["--model", "qwen2.5-0.5b", "--cp", "4", "--seq-len", "16384", "--local-budget", "2048",
                           "--reps", "2"])
    assert rc == 0
    rep = json.loads(capsys.readouterr().out.strip().splitlines()[-1])
    # rank 3 of 4 holds chunks 3 and 4 of 8: prefix = 5 chunks, 2 of them its own
    assert rep["exchanged_rows"] == 3 * (16384 // 8)
    assert rep["serial_ms"] > 0 and rep["overlapped_ms"] > 0

"""DACP and GDS end to end on the GPU: a micro-batch scheduled by the library's heuristic,
every rank's share run through the attention kernels, and the pieces put back
together and compared with the fp64 oracle of the WHOLE (unscheduled) micro-batch:
O / LSE / dQ rows come from exactly one rank; dK / dV of a distributed sequence are
the sum of the ranks' partial gradients (the reduce a real CP group would do)."""
import json

import numpy as np
import pytest

from paper_2505_19609_amd import workloads as W
from gpu_util import run_library, widen

pytestmark = pytest.mark.gpu

TOL_O, TOL_G = 2e-2, 5e-2


def _reassemble_and_compare(oracle, S, ret, N, heads, d, cut, seed, label):
    """Run every CP rank's share of the micro-batch S under the schedule `ret` through the
    attention kernels, put the pieces back together and compare them with the fp64 oracle of
    the WHOLE, unscheduled micro-batch."""
    from paper_2505_19609_amd import binding as B
    Hq, Hkv = heads
    S = [int(x) for x in S]
    whole = W.Workload("whole", S, [1] * len(S), [0] * len(S), Hq, Hkv, d, d ** -0.5, seed)
    T = sum(S)
    vals = W.make_values(whole, T, T)
    f = widen(vals)
    desc = oracle.ranges(whole.seq_len, whole.shard_degree, whole.shard_index)
    O, LSE = oracle.attention_fwd(f["q"], f["k"], f["v"], desc, whole.softmax_scale)
    dQ, dK, dV, _ = oracle.attention_bwd(f["q"], f["k"], f["v"], f["do"], desc, whole.softmax_scale)
    start = np.concatenate([[0], np.cumsum(S)])

    o = np.full(O.shape, np.nan); lse = np.full(LSE.shape, np.nan); dq = np.full(dQ.shape, np.nan)
    dk = np.zeros(dK.shape); dv = np.zeros(dV.shape)
    seen_q = np.zeros(T, np.int32)
    for j in range(N):
        seq, deg, idx, src = B.skrull_dacp_rank_batch(S, ret, N, j)
        if len(seq) == 0:
            continue
        qrows, krows = [], []
        cuts = [cut if g > 1 else 0 for g in deg]
        for s, g, i, k, z in zip(seq, deg, idx, src, cuts):
            if z:   # chunks i and 2g-1-i of 2g
                parts = [((c * s) // (2 * g), ((c + 1) * s) // (2 * g)) for c in (i, 2 * g - 1 - i)]
            else:
                parts = [((i * s) // g, ((i + 1) * s) // g)]
            for b, e in parts:
                qrows.append(np.arange(start[k] + b, start[k] + e))
            krows.append(np.arange(start[k], start[k] + parts[-1][1]))
        qrows, krows = np.concatenate(qrows), np.concatenate(krows)
        rv = {"q": vals["q"][qrows], "do": vals["do"][qrows], "k": vals["k"][krows], "v": vals["v"][krows]}
        w = W.Workload(f"rank{j}", list(seq), list(deg), list(idx), Hq, Hkv, d, d ** -0.5, 0, shard_cut=cuts)
        out = run_library(w, vals=rv)
        assert out["plan"].total_q == len(qrows) and out["plan"].total_k == len(krows)
        o[qrows], dq[qrows], lse[:, qrows] = out["o"], out["dq"], out["lse"]
        np.add.at(dk, krows, out["dk"])
        np.add.at(dv, krows, out["dv"])
        seen_q[qrows] += 1
        out["plan"].destroy()
    assert (seen_q == 1).all()  # Eq. 7: every token's query row lives on exactly one rank
    for name, got, ref, tol in (("O", o, O, TOL_O), ("LSE", lse, LSE, TOL_O), ("dQ", dq, dQ, TOL_G),
                                ("dK", dk, dK, TOL_G), ("dV", dv, dV, TOL_G)):
        err = np.abs(got - ref).max()
        print(f"{label} {name}: max-abs {err:.4g} (tol {tol})")
        assert np.isfinite(got).all() and err <= tol, (name, err)


@pytest.mark.parametrize("cut", [0, 1])
@pytest.mark.parametrize("N,C,heads,d", [(4, 2000, (4, 2), 64), (3, 2400, (6, 2), 128)])
def test_scheduled_ranks_reassemble_to_oracle(oracle, N, C, heads, d, cut):
    from paper_2505_19609_amd import binding as B
    from oracle import dacp as OD

    S = [700, 50, 1500, 300, 64, 2048, 33, 900, 17, 411]
    Hq, Hkv = heads
    ret = B.skrull_dacp_schedule(S, C, N, Hq * d, Hkv * d)
    assert list(ret) == OD.dacp_schedule(S, C, N, Hq * d, Hkv * d)
    assert (ret == -1).any() and (ret >= 0).any()
    _reassemble_and_compare(oracle, S, ret, N, heads, d, cut, 4242, f"N={N}")


@pytest.mark.parametrize("cut", [0, 1])
def test_gds_iteration_matches_oracle_schedule_and_attention(oracle, cut):
    """Alg. 2 end to end: the library's GDS schedule of a global batch (bin-packing over the
    DP ranks, stride-interleaved micro-batches, DACP decisions) equals the oracle's decision
    for decision, and every micro-batch of every DP rank, run rank by rank through the
    attention kernels under that schedule, reassembles to the fp64 oracle's attention."""
    from paper_2505_19609_amd import binding as B
    from oracle import gds as OG

    rng = np.random.Generator(np.random.PCG64(77 + cut))
    S = [int(x) for x in np.concatenate([rng.integers(16, 700, 18), rng.integers(900, 2000, 6)])]
    rng.shuffle(S)
    C, N, ws, heads, d = 1024, 2, 2, (4, 2), 64
    h, hkv = heads[0] * d, heads[1] * d
    n_mb = n_dist = 0
    for r in range(ws):
        want = OG.gds_schedule(S, C, N, ws, r, h, hkv)
        assert want is not None
        bins, mb, ret, m = B.skrull_gds_schedule(S, C, N, ws, r, h, hkv)
        assert list(bins) == want[0] and m == len(want[1])
        for j, wmb in enumerate(want[1]):
            members = B.skrull_gds_micro_batch(S, mb, j)
            assert [(int(k), int(ret[k])) for k in members] == wmb          # paper Alg. 2, via Alg. 1
            assert sum(S[k] for k in members) <= C * N
            n_dist += int((ret[members] == -1).sum())
            n_mb += 1
            _reassemble_and_compare(oracle, [S[k] for k in members], ret[members], N, heads, d, cut,
                                    900 + 10 * r + j, f"dp{r} mb{j}")
    assert n_mb > ws and n_dist > 0      # several micro-batches per rank, some sequences distributed


def test_driver_reports_every_rank(capsys):
    from paper_2505_19609_amd import dacp_run
    rc = dacp_run.main(["--dataset", "chatqa2_long_sft", "--model", "qwen2.5-0.5b", "--cp", "4",
                        "--bucket", "16384", "--fill", "0.7", "--reps", "1", "--compare", "--seed", "3"])
    assert rc == 0
    rep = json.loads(capsys.readouterr().out.strip().splitlines()[-1])
    assert rep["cp_degree"] == 4 and len(rep["dacp"]["ranks"]) == 4 and len(rep["plain_cp"]["ranks"]) == 4
    assert rep["local_seqs"] + rep["distributed_seqs"] == rep["num_seqs"]
    # Eq. 7/8: all tokens are placed, none twice, no rank over its bucket
    assert sum(r["tokens"] for r in rep["dacp"]["ranks"]) == rep["tokens"]
    assert sum(r["tokens"] for r in rep["plain_cp"]["ranks"]) == rep["tokens"]
    assert max(r["tokens"] for r in rep["dacp"]["ranks"]) <= rep["bucket_size"] + rep["distributed_seqs"]
    assert rep["dacp"]["max_ms"] >= rep["dacp"]["min_ms"] > 0


def test_gds_driver_runs_a_whole_iteration(capsys):
    from paper_2505_19609_amd import gds_run
    rc = gds_run.main(["--dataset", "wikipedia", "--model", "qwen2.5-0.5b", "--cp", "2", "--dp", "2",
                       "--batch-size", "12", "--bucket", "2048", "--reps", "1", "--seed", "1"])
    assert rc == 0
    rep = json.loads(capsys.readouterr().out.strip().splitlines()[-1])
    assert len(rep["dp_ranks"]) == 2
    assert sum(r["num_seqs"] for r in rep["dp_ranks"]) == rep["num_seqs"] == 24
    for r in rep["dp_ranks"]:
        assert sum(m["tokens"] for m in r["micro_batches"]) == r["tokens"]
        assert all(m["tokens"] <= 2 * 2048 for m in r["micro_batches"])   # C*N per micro-batch
        assert abs(sum(m["max_ms"] for m in r["micro_batches"]) - r["sum_max_ms"]) < 1e-2
    assert rep["iteration_ms"] == max(r["sum_max_ms"] for r in rep["dp_ranks"])


def test_calibration_fit(capsys):
    from paper_2505_19609_amd import calibrate
    rc = calibrate.main(["--model", "qwen2.5-7b", "--cp", "4", "--lengths", "512", "2048", "8192", "--reps", "2"])
    assert rc == 0
    rep = json.loads(capsys.readouterr().out.strip().splitlines()[-1])
    assert len(rep["rows"]) == 3 and rep["alpha_ms_per_flop"] > 0
    ms = [r["whole_ms"] for r in rep["rows"]]
    assert ms[0] < ms[1] < ms[2]
    # the last contiguous slice sees (2N-1) times the pairs of the first one
    assert rep["rows"][2]["slice_last_ms"] > rep["rows"][2]["slice_first_ms"]

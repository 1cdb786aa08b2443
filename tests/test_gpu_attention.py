"""Parity of the HIP forward/backward with the fp64 oracle, through the C ABI.

Tolerances are the stated ones: max-abs 2e-2 on O (and LSE), 5e-2 on dQ/dK/dV,
GPU bf16 outputs widened and compared with the unrounded fp64 oracle on the
same seeded bf16 inputs.  Two exceptions, both where gradients carry 8x the usual
softmax scale: config 1 as stated adds one spacing of bf16 relative to the element
(RTOL_8X: elements exceed 16 there and a bf16 output cannot meet 5e-2), and the
out-of-distribution stress test_extreme_logits scales the bound by that factor.  Small cases are compared exhaustively; the full-size
benchmark micro-batches on seeded samples of rows / columns that the oracle
computes one by one, plus properties that hold at any size."""
import numpy as np
import pytest

from paper_2505_19609_amd import workloads as W
from gpu_util import run_library, widen, bf16_ulp

pytestmark = pytest.mark.gpu

TOL_O, TOL_G = 2e-2, 5e-2


def _report(name, got, ref, tol, rtol=0.0):
    """Max-abs check; with ``rtol`` an element's bound is tol + rtol * |reference value|."""
    err = np.abs(got.astype(np.float64) - ref)
    if err.size == 0:
        return 0.0
    allowed = tol + rtol * np.abs(ref)
    i = np.unravel_index(np.argmax(err - allowed), err.shape)
    ulps = err[i] / bf16_ulp(ref[i])
    msg = (f"{name}: max-abs {err.max():.4g}; worst against its bound {err[i]:.4g} at {i} (ref {ref[i]:.6g}, "
           f"got {got[i]:.6g}, {ulps:.2f} bf16 ulp), bound {allowed[i]:.4g}")
    print(msg)
    assert np.isfinite(got).all(), f"{name}: non-finite output"
    assert err[i] <= allowed[i], msg
    return float(err[i])


# Relative part of the bound for config 1 as stated, whose dQ carries 8x the usual softmax
# scale: elements reach |x| > 16 and the stated max-abs
# 5e-2 is below the spacing of the bf16 output (0.125): one spacing of bf16 relative to the
# reference value, 2^-7.  Three bf16 roundings of relative size 2^-9 lie on the path of a
# gradient element (the forward's O, from which D = dO.O is formed; dS before the second
# product; the output itself), and in a query row that sees only a few keys nothing averages
# them out.  Observed worst (config 1 as stated): 0.0745 on dQ = -15.637 and 0.054 on -7.836,
# both in a row with three keys; 0.0888 on |dQ| > 16.  Elements of ordinary size keep 5e-2.
RTOL_8X = 2.0 ** -7


def _exhaustive(oracle, w, block_m=0, block_n=0, rtol=0.0, head_split=0, wg_query_rows=0, keep=False):
    out = run_library(w, block_m, block_n, head_split=head_split, wg_query_rows=wg_query_rows)
    if wg_query_rows:
        assert out["plan"].info.wg_query_rows == wg_query_rows
    f = widen(out["vals"])
    desc = oracle.ranges(w.seq_len, w.shard_degree, w.shard_index, w.shard_cut)
    O, LSE = oracle.attention_fwd(f["q"], f["k"], f["v"], desc, w.softmax_scale)
    dQ, dK, dV, _ = oracle.attention_bwd(f["q"], f["k"], f["v"], f["do"], desc, w.softmax_scale)
    _report("O", out["o"], O, TOL_O)
    _report("LSE", out["lse"], LSE, TOL_O)
    _report("dQ", out["dq"], dQ, TOL_G, rtol)
    _report("dK", out["dk"], dK, TOL_G, rtol)
    _report("dV", out["dv"], dV, TOL_G, rtol)
    if not keep:
        out["plan"].destroy()
    return out


def test_config1_tiny_literal(oracle):
    """Config 1 as stated: Q pre-scaled by 1/8 in the data, no further scale.  dQ is then the
    gradient w.r.t. the pre-scaled Q, 8x the gradient w.r.t. the N(0,1) draw, and reaches
    |dQ| = 21.9; rounding the exact result to bf16 alone errs by 0.060 there
    (test_config1_dq_rounding_floor).  Every element is held to the stated 5e-2 plus one
    spacing of bf16 relative to its reference value (RTOL_8X)."""
    _exhaustive(oracle, W.config(1), rtol=RTOL_8X)


def test_config1_tiny_scale_in_kernel(oracle):
    """Same lengths and draws, the 1/sqrt(64) applied as softmax_scale inside the kernels
    instead: every stated tolerance applies as is.  And the literal variant's results are the
    SAME BITS (dQ times 8: the pre-scaling by a power of two is exact in bf16 and commutes
    with every rounding), so the literal dQ is exactly as accurate as this one."""
    w = W.config(1)
    w.q_prescale, w.softmax_scale = 1.0, 0.125
    a = _exhaustive(oracle, w)
    b = run_library(W.config(1))
    for n in ("o", "lse", "dk", "dv"):
        assert np.array_equal(a[n], b[n]), n
    assert np.array_equal(8.0 * a["dq"], b["dq"])
    b["plan"].destroy()


def test_config2_qwen05b(oracle):
    _exhaustive(oracle, W.config(2))


EDGE = {
    "single_tokens": ([1, 1, 2], [1, 1, 1], [0, 0, 0]),
    "around_32": ([31, 32, 33], [1] * 3, [0] * 3),
    "around_64": ([63, 64, 65], [1] * 3, [0] * 3),
    "around_128": ([127, 128, 129, 130], [1] * 4, [0] * 4),
    "around_256": ([255, 257], [1] * 2, [0] * 2),
    "ragged_shards": ([1000, 999, 130, 70], [3, 7, 2, 70], [1, 6, 1, 69]),
    "first_shards": ([900, 333], [4, 2], [0, 0]),
}


@pytest.mark.parametrize("name", sorted(EDGE))
@pytest.mark.parametrize("heads,d,wg,hs", [((4, 4), 64, 0, 0), ((6, 2), 128, 256, 3), ((8, 1), 128, 128, 0),
                                           ((14, 2), 64, 256, 7)])
def test_every_store_stays_inside_its_tensor(name, heads, d, wg, hs):
    """Outputs and workspace sit between marked margins: a store of a row block that ran past the
    end of a ragged micro-batch (or before its start) would change them.  Every element inside
    is written (no NaN of the pre-fill is left) and the result equals the unguarded run's bits."""
    S, N, R = EDGE[name]
    w = W.Workload(f"guard_{name}", S, N, R, heads[0], heads[1], d, d ** -0.5, 77)
    a = run_library(w, head_split=hs, wg_query_rows=wg, guard=True)
    assert a["margins"] == [], a["margins"]
    b = run_library(w, head_split=hs, wg_query_rows=wg)
    for n in ("o", "lse", "dq", "dk", "dv"):
        assert np.isfinite(a[n]).all(), n
        assert np.array_equal(a[n], b[n]), n
    a["plan"].destroy()
    b["plan"].destroy()


@pytest.mark.parametrize("name", sorted(EDGE))
@pytest.mark.parametrize("heads,d", [((4, 4), 64), ((6, 2), 128), ((8, 1), 128), ((2, 1), 64)])
def test_edge_cases(oracle, name, heads, d):
    S, N, R = EDGE[name]
    w = W.Workload(name, S, N, R, heads[0], heads[1], d, d ** -0.5, 500 + len(S) + d)
    _exhaustive(oracle, w)


@pytest.mark.parametrize("heads", [(5, 5), (16, 1), (24, 8), (40, 8), (9, 9), (10, 5)])
def test_head_configurations(oracle, heads):
    """Head counts that are not powers of two or do not divide the 8 dies the blocks are
    dealt to (the block-to-head mapping must stay a bijection whatever Hkv is)."""
    d = 64 if heads[0] % 2 else 128
    w = W.Workload(f"heads{heads[0]}_{heads[1]}", [300, 65, 1, 190], [1, 1, 1, 2], [0, 0, 0, 1],
                   heads[0], heads[1], d, d ** -0.5, 900 + heads[0])
    _exhaustive(oracle, w)


def test_thousands_of_tiny_sequences(oracle):
    """3,000 sequences of 1 to 16 tokens: every work item is a sliver of one tile."""
    rng = np.random.Generator(np.random.PCG64(3000))
    S = [int(x) for x in rng.integers(1, 17, 3000)]
    w = W.Workload("tiny3000", S, [1] * len(S), [0] * len(S), 4, 2, 64, 0.125, 3001)
    _exhaustive(oracle, w)


@pytest.mark.parametrize("scale,d", [(1.0, 64), (0.75, 128), (0.002, 128)])
def test_extreme_logits(oracle, scale, d):
    """Scores far outside the usual range: with softmax_scale 1 (0.75) on N(0,1) data of
    head_dim 64 (128) they have a standard deviation of 8 and single rows reach +-40,
    so probabilities span e^80 and the running maximum has to move; with 0.002 the
    softmax is almost uniform.  (The forward's bound on the scores of a row may lag behind them by up to 2^10.)"""
    w = W.Workload(f"logits{scale}", [700, 1300, 64], [1, 1, 1], [0, 0, 0], 4, 2, d, scale, 4242)
    out = run_library(w)
    f = widen(out["vals"])
    desc = oracle.ranges(w.seq_len, w.shard_degree, w.shard_index)
    O, LSE = oracle.attention_fwd(f["q"], f["k"], f["v"], desc, w.softmax_scale)
    dQ, dK, dV, _ = oracle.attention_bwd(f["q"], f["k"], f["v"], f["do"], desc, w.softmax_scale)
    _report("O", out["o"], O, TOL_O)
    _report("LSE", out["lse"], LSE, TOL_O)
    # A stress case outside the stated configurations: dQ and dK carry the factor softmax_scale,
    # here k = scale * sqrt(d) = 8 (6) times the usual 1/sqrt(d), and every absolute error of
    # the bf16 path grows with it, also on elements that are themselves near zero (0.166 on a
    # dQ of -0.006 whose row has terms of size 10).  The stated bound is therefore applied to
    # the gradients divided by k, i.e. 5e-2 * k on the outputs; O, LSE, dV keep theirs.
    k = max(1.0, scale * d ** 0.5)
    _report("dQ", out["dq"] / k, dQ / k, TOL_G)
    _report("dK", out["dk"] / k, dK / k, TOL_G)
    _report("dV", out["dv"], dV, TOL_G)
    out["plan"].destroy()


@pytest.mark.parametrize("bm,bn", [(64, 64), (64, 256), (256, 64), (256, 256), (128, 64), (0, 192), (64, 192)])
@pytest.mark.parametrize("d", [64, 128])
def test_block_sizes(oracle, bm, bn, d):
    w = W.Workload("blocks", [700, 129, 1030, 64], [1, 1, 2, 1], [0, 0, 1, 0], 4, 2, d, d ** -0.5, 77)
    _exhaustive(oracle, w, bm, bn)


@pytest.mark.parametrize("index", [0, 7])
def test_scaled_down_shard_twin(oracle, index):
    """Structure of config 4 (one sequence sharded 8 ways + short local ones) at a
    size the oracle covers exhaustively; every tile class occurs (interior,
    diagonal, shard-offset diagonal, ragged tail)."""
    _exhaustive(oracle, W.scaled_shard_twin(seq_len=8192, degree=8, index=index))


def test_determinism_and_plan_reuse(oracle):
    """No atomics anywhere: two runs are bit-identical; a plan serves many calls."""
    import torch
    from paper_2505_19609_amd import binding as B
    w = W.config(2)
    a = run_library(w, keep_device=True)
    dev, res, plan = a["dev_in"], a["dev"], a["plan"]
    o2, lse2 = torch.empty_like(res["o"]), torch.empty_like(res["lse"])
    dq2, dk2, dv2 = torch.empty_like(res["dq"]), torch.empty_like(res["dk"]), torch.empty_like(res["dv"])
    ws = torch.empty(int(plan.bwd_workspace_bytes), dtype=torch.uint8, device="cuda")
    B.skrull_attn_fwd(plan, dev["q"], dev["k"], dev["v"], o2, lse2)
    B.skrull_attn_bwd(plan, dev["q"], dev["k"], dev["v"], o2, lse2, dev["do"], dq2, dk2, dv2, ws)
    torch.cuda.synchronize()
    for x, y in ((res["o"], o2), (res["lse"], lse2), (res["dq"], dq2), (res["dk"], dk2), (res["dv"], dv2)):
        assert torch.equal(x.view(torch.int16) if x.dtype == torch.bfloat16 else x,
                           y.view(torch.int16) if y.dtype == torch.bfloat16 else y)
    plan.destroy()


@pytest.mark.parametrize("d,cut", [(64, 0), (128, 1)])
def test_nan_in_one_sequence_stays_there(oracle, d, cut):
    """No cross-sequence leakage, the strict way: every value of one sequence is NaN, and the
    results of all the others are bit-identical to a run on clean data (a probability of
    zero times a NaN would still be a NaN, so no tile may even contain a neighbour's rows)."""
    S, N, R = [200, 333, 70, 129, 1, 600], [1, 1, 1, 1, 1, 3], [0, 0, 0, 0, 0, 1]
    Z = [0, 0, 0, 0, 0, cut]
    w = W.Workload("poison", S, N, R, 6, 2, d, d ** -0.5, 1234, shard_cut=Z)
    clean = run_library(w)
    desc = oracle.ranges(S, N, R, Z)
    nan_bits = np.uint16(0x7FC0)
    for victim in (2, 5, 0):
        vals = {n: a.copy() for n, a in clean["vals"].items()}
        # rows of the poisoned sequence in the packed tensors
        q_lo, q_hi = _rows_of(desc, victim, "cu_q")
        k_lo, k_hi = _rows_of(desc, victim, "cu_k")
        for n in ("q", "do"):
            vals[n][q_lo:q_hi] = nan_bits
        for n in ("k", "v"):
            vals[n][k_lo:k_hi] = nan_bits
        out = run_library(w, vals=vals)
        for n, (lo, hi) in (("o", (q_lo, q_hi)), ("dq", (q_lo, q_hi)), ("dk", (k_lo, k_hi)), ("dv", (k_lo, k_hi))):
            keep = np.ones(out[n].shape[0], bool)
            keep[lo:hi] = False
            assert np.array_equal(out[n][keep], clean[n][keep]), (victim, n)
        keep = np.ones(out["lse"].shape[1], bool)
        keep[q_lo:q_hi] = False
        assert np.array_equal(out["lse"][:, keep], clean["lse"][:, keep]), (victim, "lse")
        out["plan"].destroy()
    clean["plan"].destroy()


def _rows_of(desc, k, cu):
    """Packed row range [lo, hi) of sequence k (its one or two query segments / its prefix)."""
    segs = [i for i, q in enumerate(_segment_owner(desc)) if q == k]
    if cu == "cu_q":
        return int(desc["cu_q"][segs[0]]), int(desc["cu_q"][segs[-1] + 1])
    return int(desc["cu_k"][segs[0]]), int(desc["cu_k"][segs[-1] + 1])


def _segment_owner(desc):
    """Sequence index of every query segment: a segment that shares the prefix of the one
    before it belongs to the same sequence."""
    owner, k = [], -1
    for sh in desc["shares_kv"]:
        if not sh:
            k += 1
        owner.append(k)
    return owner


def test_sequence_order_permutes_outputs(oracle):
    """The library is agnostic to the order of sequences in the packed batch."""
    S, N, R = [300, 64, 1000, 129], [1, 1, 4, 1], [0, 0, 2, 0]
    w = W.Workload("perm", S, N, R, 4, 2, 128, 128 ** -0.5, 91)
    a = run_library(w)
    desc = oracle.ranges(S, N, R)
    perm = [2, 0, 3, 1]
    w2 = W.Workload("perm2", [S[i] for i in perm], [N[i] for i in perm], [R[i] for i in perm],
                    4, 2, 128, 128 ** -0.5, 91)
    desc2 = oracle.ranges(w2.seq_len, w2.shard_degree, w2.shard_index)
    vals2 = {}
    for n, cu, cu2 in (("q", "cu_q", "cu_q"), ("do", "cu_q", "cu_q"), ("k", "cu_k", "cu_k"), ("v", "cu_k", "cu_k")):
        parts = [a["vals"][n][desc[cu][i]:desc[cu][i + 1]] for i in perm]
        vals2[n] = np.concatenate(parts)
    b = run_library(w2, vals=vals2)
    for n, cu in (("o", "cu_q"), ("dq", "cu_q"), ("dk", "cu_k"), ("dv", "cu_k")):
        for pos, i in enumerate(perm):
            x = a[n][desc[cu][i]:desc[cu][i + 1]]
            y = b[n][desc2[cu][pos]:desc2[cu][pos + 1]]
            assert np.array_equal(x, y), (n, i)


# ---------------------------------------------------------------------------
# full-size micro-batches: sampled oracle parity + size-independent properties
# ---------------------------------------------------------------------------
def _by_kv_head(fn, f, names, desc, scale, ent, g):
    """oracle.fwd_rows / oracle.bwd_dq_rows on the (segment, head, row) entries `ent`, one KV head
    at a time on contiguous copies of that head's K and V and of its g query heads.  Only the
    packing of the inputs changes (a key row is then 4*d bytes from the next instead of
    4*d*Hkv, which the host's caches and prefetchers like 2-3x better on long prefixes); the
    oracle does the same arithmetic in the same order and returns the same bits."""
    a = np.zeros((len(ent[0]), f["q"].shape[2]))
    b = np.zeros(len(ent[0]))
    for c in np.unique(ent[1] // g):
        sel = np.nonzero(ent[1] // g == c)[0]
        sub = (ent[0][sel], (ent[1][sel] - c * g).astype(np.int32), ent[2][sel])
        args = [np.ascontiguousarray(f[n][:, c * g:(c + 1) * g] if n in ("q", "do") else f[n][:, c:c + 1])
                for n in names]
        a[sel], b[sel] = fn(*args, desc, scale, sub)
    return a, b


def _progress(capsys, msg):
    """One line straight to the terminal (past pytest's capture): a full-size case keeps the
    oracle busy for minutes, and a run that prints nothing that long is taken to be hung."""
    if capsys is None:
        print(msg, flush=True)
    else:
        with capsys.disabled():
            print(msg, flush=True)


# Largest whole forward of one KV group that the oracle is asked for, in (query row, key, head)
# triples, unless a test names its own: config 3's long sequence (1.2e9) and the first slice
# of config 4 fit.  A sequence above it (the 131,072-token prefix of config 4's last slice costs
# 8e9, minutes on the host cores) has its key columns drawn over as long a tail of the prefix
# as the cap affords; its early key blocks run the same chains, only longer, and are covered
# whole at a quarter of the length (test_config4_quarter_twin).
GROUP_COST_CAP = 2.0e9


def _sampled(oracle, w, rows_per_long, cols_per_long, seed, exhaustive_below=400, vals=None,
             heads_per_row=None, wg_query_rows=0, window=None, capsys=None, group_cap=None,
             slice_group_cap=None, few_heads_from=0):
    """Full-size parity on samples the oracle computes one by one.

    Every segment of at most ``exhaustive_below`` query rows: all rows x all heads (O, LSE, dQ)
    and all of its key columns x all KV heads (dK, dV).  Every longer sequence: ``rows_per_long``
    seeded query rows plus fixed ones at tile edges x every head (O, LSE, dQ); and ONE seeded KV
    group for which the oracle runs the whole forward (LSE and D = dO.O of every query row of
    the group's heads, all of them also compared as O / LSE), so that dK / dV can be compared
    on ``cols_per_long`` seeded key columns drawn over the WHOLE prefix plus fixed ones in the
    first key blocks, at the chunk boundaries and on the diagonal.  A sequence whose whole
    forward exceeds GROUP_COST_CAP gets its columns from the longest tail of the prefix that
    fits the cap (``group_cap``, or ``slice_group_cap`` for a slice that does not start at
    position 0).  ``heads_per_row`` limits the sampled rows of segments whose prefix has at
    least ``few_heads_from`` keys to that many seeded heads each.  ``window``, if given, instead limits the columns of long sequences to the
    last ``window`` keys (then only the last rows' LSE / D are needed): the mode of the
    address-range test below."""
    import time
    t_start = time.time()
    out = run_library(w, vals=vals, wg_query_rows=wg_query_rows)
    f = widen(out["vals"])
    desc = oracle.ranges(w.seq_len, w.shard_degree, w.shard_index, w.shard_cut)
    Hq, Hkv, d = w.num_q_heads, w.num_kv_heads, w.head_dim
    g = Hq // Hkv
    ns = desc["num_seqs"]
    rng = np.random.Generator(np.random.PCG64(seed))
    owner = _segment_owner(desc)
    seqs = [[s for s in range(ns) if owner[s] == k] for k in range(owner[-1] + 1)]
    is_long = [any(int(desc["q_len"][s]) > exhaustive_below for s in segs) for segs in seqs]
    Tq = desc["total_q"]
    LSEf = np.full((Hq, Tq), np.nan)
    Df = np.full((Hq, Tq), np.nan)

    def edges(n, marks):
        """positions around the given marks and 32/64/128-row tile edges, inside [0, n)"""
        e = [m + o for m in marks for o in (-129, -128, -65, -64, -33, -32, -2, -1, 0, 1, 31, 32, 63, 64,
                                            127, 128, 129, 191, 192, 255, 256)]
        return np.array(sorted({x for x in e if 0 <= x < n}), np.int64)

    # --- rows: O, LSE, dQ ---
    es, eh, ei = [], [], []
    for k, segs in enumerate(seqs):
        for s in segs:
            ql = int(desc["q_len"][s])
            if not is_long[k]:
                rows = np.arange(ql)
            else:
                rows = np.unique(np.concatenate([edges(ql, [0, ql]),
                                                 rng.choice(ql, min(ql, rows_per_long), replace=False)]))
            for i in rows:
                heads = np.arange(Hq)
                if is_long[k] and heads_per_row is not None and int(desc["kv_len"][s]) >= few_heads_from:
                    heads = np.sort(rng.choice(Hq, heads_per_row, replace=False))
                es.append(np.full(len(heads), s)); eh.append(heads); ei.append(np.full(len(heads), i))
    ent = tuple(np.concatenate(x).astype(np.int32) for x in (es, eh, ei))
    prow = desc["cu_q"][ent[0]] + ent[2]
    o_ref, lse_ref = _by_kv_head(oracle.fwd_rows, f, ("q", "k", "v"), desc, w.softmax_scale, ent, g)
    _progress(capsys, f"  [{w.name}: oracle forward of {len(prow)} sampled rows done, {time.time() - t_start:.0f} s]")
    dq_ref, d_ref = _by_kv_head(oracle.bwd_dq_rows, f, ("q", "k", "v", "do"), desc, w.softmax_scale, ent, g)
    _progress(capsys, f"  [{w.name}: oracle dQ of the sampled rows done, {time.time() - t_start:.0f} s]")
    LSEf[ent[1], prow] = lse_ref
    Df[ent[1], prow] = d_ref
    print(f"{w.name}: checked {len(prow)} (row, head) entries of O/LSE/dQ "
          f"({sum(is_long)} long sequences: >= {rows_per_long} seeded rows each x {Hq} heads"
          + (f", {heads_per_row} seeded heads per row where the prefix has {few_heads_from} keys or more"
             if heads_per_row else "") + ")")
    _report("O", out["o"][prow, ent[1]], o_ref, TOL_O)
    _report("LSE", out["lse"][ent[1], prow], lse_ref, TOL_O)
    _report("dQ", out["dq"][prow, ent[1]], dq_ref, TOL_G)

    # --- LSE and D of one KV group of every long sequence, over all the rows its sampled
    #     columns can see (the whole sequence unless `window` is given) ---
    group_of, col_lo = {}, {}
    chunks = []                          # one (segment, head, rows) piece of oracle work at a time
    for k, segs in enumerate(seqs):
        if not is_long[k]:
            continue
        c = int(rng.integers(0, Hkv))
        group_of[k] = c
        kvl = int(desc["kv_len"][segs[-1]])
        if window is not None:
            col_lo[k] = max(0, kvl - window)
        else:
            # rows (of all the segments) from the end of the sequence backwards until the cap:
            # the row at position p costs (p + 1) * g
            pos = np.concatenate([int(desc["q_begin"][s]) + np.arange(int(desc["q_len"][s])) for s in segs])
            cost = np.cumsum((pos[::-1] + 1.0) * g)
            cap = group_cap or GROUP_COST_CAP
            if int(desc["q_begin"][segs[-1]]) > 0 and slice_group_cap:   # a slice that sees a long prefix
                cap = slice_group_cap
            n_rows = int(np.searchsorted(cost, cap, side="right"))
            col_lo[k] = 0 if n_rows >= len(pos) else int(pos[len(pos) - n_rows])
        for s in segs:
            ql, qb = int(desc["q_len"][s]), int(desc["q_begin"][s])
            ii = np.arange(max(0, col_lo[k] - qb), ql)
            for hh in range(c * g, (c + 1) * g):
                chunks.append((s, hh, ii))
    n_grp = 0
    for s, hh, ii in chunks:
        if len(ii) == 0:
            continue
        grp = (np.full(len(ii), s, np.int32), np.full(len(ii), hh, np.int32), ii.astype(np.int32))
        grow = desc["cu_q"][s] + ii
        o_g, lse_g = _by_kv_head(oracle.fwd_rows, f, ("q", "k", "v"), desc, w.softmax_scale, grp, g)
        LSEf[hh, grow] = lse_g
        Df[hh, grow] = oracle.delta_rows(f["do"][grow, hh], o_g)
        _report(f"O (segment {s}, head {hh}, {len(ii)} rows)", out["o"][grow, hh], o_g, TOL_O)
        _report(f"LSE (segment {s}, head {hh})", out["lse"][hh, grow], lse_g, TOL_O)
        n_grp += len(ii)
        if len(ii) * (int(desc["q_begin"][s]) + ii[-1]) > 2e8:
            _progress(capsys, f"  [{w.name}: oracle forward of segment {s}, head {hh}, rows {ii[0]}..{ii[-1]} done, "
                              f"{time.time() - t_start:.0f} s]")
    if n_grp:
        print(f"{w.name}: forward of one KV group per long sequence: {n_grp} (row, head) entries of O/LSE checked")

    # --- columns: dK, dV ---
    cs, cc, cj, ct = [], [], [], []      # (segment, kv head, key position) -> target slot
    tk, tc = [], []                      # target slots: packed key row, kv head
    n_long_cols = 0
    for k, segs in enumerate(seqs):
        last = segs[-1]
        kvl, base = int(desc["kv_len"][last]), int(desc["cu_k"][last])
        if not is_long[k]:
            ql, qb = int(desc["q_len"][last]), int(desc["q_begin"][segs[0]])
            groups = range(Hkv)
            cols = np.arange(0 if kvl <= 4096 else kvl - ql, kvl)
        else:
            groups = [group_of[k]]
            if window is None:
                lo = col_lo[k]
                marks = [lo, kvl] + [int(desc["q_begin"][s]) for s in segs] + [int(desc["kv_len"][s]) for s in segs]
                cols = np.unique(np.concatenate([edges(kvl, marks),
                                                 lo + rng.choice(kvl - lo, min(kvl - lo, cols_per_long), replace=False)]))
                cols = cols[cols >= lo]
            else:
                cols = np.arange(col_lo[k], kvl)
            n_long_cols += len(cols)
        for c in groups:
            slot0 = len(tk)
            tk.extend(base + cols); tc.extend([c] * len(cols))
            for s in segs:
                vis = cols < int(desc["kv_len"][s])
                cs.append(np.full(int(vis.sum()), s)); cc.append(np.full(int(vis.sum()), c)); cj.append(cols[vis])
                ct.append(slot0 + np.nonzero(vis)[0])
    cent = tuple(np.concatenate(x).astype(np.int32) for x in (cs, cc, cj))
    slot = np.concatenate(ct)
    _progress(capsys, f"  [{w.name}: oracle rows and forward done, {time.time() - t_start:.0f} s]")
    dk_e, dv_e = oracle.bwd_dkv_cols(f["q"], f["k"], f["v"], f["do"], LSEf, Df, desc, w.softmax_scale, cent)
    _progress(capsys, f"  [{w.name}: oracle key columns done, {time.time() - t_start:.0f} s]")
    assert np.isfinite(dk_e).all() and np.isfinite(dv_e).all()
    tk, tc = np.array(tk), np.array(tc)
    dk_ref, dv_ref = np.zeros((len(tk), d)), np.zeros((len(tk), d))
    np.add.at(dk_ref, slot, dk_e)    # the two chunks of a two-chunk cut both reach the shared prefix
    np.add.at(dv_ref, slot, dv_e)
    span = "; ".join(f"sequence {k}: keys {col_lo[k]}..{int(desc['kv_len'][seqs[k][-1]]) - 1}" for k in sorted(col_lo)
                     if int(desc["kv_len"][seqs[k][-1]]) > 4096)
    print(f"{w.name}: checked {len(tk)} (key, kv head) entries of dK/dV, {n_long_cols} of them columns of "
          f"long sequences ({span})")
    _report("dK", out["dk"][tk, tc], dk_ref, TOL_G)
    _report("dV", out["dv"][tk, tc], dv_ref, TOL_G)

    # --- properties that hold at any size, on ALL outputs ---
    for n in ("o", "lse", "dq", "dk", "dv"):
        assert np.isfinite(out[n]).all(), n
    def dots(x, y):
        """Per head: sum of x*y over rows and head dims, accumulated in fp64, and an
        estimate of the sum of (x*y)^2 (from every st-th row when there are many)."""
        st = max(1, x.shape[0] // 65536)
        xs, ys = x[::st], y[::st]
        return (np.einsum("ihd,ihd->h", x, y, dtype=np.float64),
                st * np.einsum("ihd,ihd,ihd,ihd->h", xs, ys, xs, ys, dtype=np.float64))

    for segs in seqs:
        qs, qe = desc["cu_q"][segs[0]], desc["cu_q"][segs[-1] + 1]
        ks, ke = desc["cu_k"][segs[-1]], desc["cu_k"][segs[-1] + 1]
        per_group = lambda t: t.reshape(Hkv, g).sum(axis=1)  # noqa: E731  (query heads of one KV head are adjacent)
        tq, tq2 = (per_group(t) for t in dots(out["dq"][qs:qe], f["q"][qs:qe]))
        tk_, tk2 = dots(out["dk"][ks:ke], f["k"][ks:ke])
        tv, tv2 = dots(out["dv"][ks:ke], f["v"][ks:ke])
        to, to2 = (per_group(t) for t in dots(out["o"][qs:qe], f["do"][qs:qe]))
        for c in range(Hkv):
            # scale invariance of q.k: sum_i dQ_i.Q_i == sum_j dK_j.K_j per (sequence, group)
            noise = 2.0 ** -8 * np.sqrt(tq2[c] + tk2[c])
            assert abs(tq[c] - tk_[c]) <= 8 * noise + 1e-3, (segs, c, tq[c], tk_[c], noise)
            # O = P V  =>  sum_j dV_j.V_j == sum_i dO_i.O_i
            noise = 2.0 ** -8 * np.sqrt(tv2[c] + to2[c])
            assert abs(tv[c] - to[c]) <= 8 * noise + 1e-3, (segs, c, tv[c], to[c], noise)
    out["plan"].destroy()


# Sizes of the samples (the rule: at least 256 seeded query rows of every head and at least
# 256 seeded key columns of one KV group per long sequence).
ROWS, COLS = 256, 256


@pytest.mark.timeout(600)
def test_config3_llama8b_sampled(oracle, capsys):
    _sampled(oracle, W.config(3), ROWS, COLS, seed=303, capsys=capsys)


@pytest.mark.timeout(600)
def test_config4_shard7_sampled(oracle, capsys):
    """Every query row of this slice sees 114,688 to 131,072 keys; its key columns come from the
    last 7,865 keys of the prefix (what 4e9 row-key-head triples of oracle forward afford)."""
    _sampled(oracle, W.config(4), ROWS, COLS, seed=404, capsys=capsys, slice_group_cap=4.0e9)


@pytest.mark.timeout(600)
def test_config4_shard0_sampled(oracle, capsys):
    _sampled(oracle, W.config(4, shard_index=0), ROWS, COLS, seed=405, capsys=capsys)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("index,cut", [(7, 0), (2, 1)])
def test_config4_quarter_twin(oracle, capsys, index, cut):
    """Config 4 at a quarter of its length (32,768 tokens, 8 ranks, the same heads and short
    sequences): the last contiguous slice, and rank 2 of the balanced cut (chunks 2 and 13 of
    16), with key columns over the WHOLE prefix, chunk boundaries included."""
    w = W.config(4, shard_index=index)
    w.seq_len[0] = 32768
    w.shard_cut = [cut] + [0] * (len(w.seq_len) - 1)
    w.name = f"config4_quarter_rank{index}_cut{cut}"
    _sampled(oracle, w, ROWS, COLS, seed=407 + cut, capsys=capsys)


@pytest.mark.timeout(600)
def test_config4_two_chunk_rank2_sampled(oracle, capsys):
    """Config 4's micro-batch with the 131,072-token sequence cut the balanced way (rank 2 of
    8 holds chunks 2 and 13 of 16, 8,192 rows each, on a prefix of 114,688 keys): key columns
    from the tail of the prefix that the cap affords, which spans the late chunk's boundary."""
    w = W.config(4, shard_index=2)
    w.shard_cut = [1] + [0] * (len(w.seq_len) - 1)
    w.name += "_two_chunks"
    _sampled(oracle, w, ROWS, COLS, seed=406, capsys=capsys, slice_group_cap=3.0e9)


@pytest.mark.timeout(800)
def test_config5_qwen7b_sampled(oracle, capsys):
    """The 38,365-token local sequence gets the whole forward of one KV group (7 query heads,
    5.2e9) and key columns over its whole prefix; the slice 3 of 4 of the 65,536-token sequence
    a tail of its prefix."""
    _sampled(oracle, W.config(5), ROWS, COLS, seed=505, capsys=capsys, group_cap=5.5e9, slice_group_cap=2.0e9)


@pytest.mark.timeout(400)
@pytest.mark.parametrize("wg_query_rows", [128, 256])
def test_byte_offsets_past_2_31_sampled(oracle, wg_query_rows):
    """One 270,000-token sequence with 32 heads of 128 on both sides: rows of 8 KB, so
    the kernels' 32-bit tile offsets into Q, dO, K and V pass 2^31 (at row 262,144) and
    end near 2.2e9.  Values are drawn on the GPU (seeded) because the numpy generator
    would take minutes for 4.4e9 numbers; the oracle gets the same bits."""
    import torch
    S, H, d = 270_000, 32, 128
    w = W.Workload("long270k_mha", [S], [1], [0], H, H, d, d ** -0.5, 0)
    gen = torch.Generator(device="cuda").manual_seed(2_700)
    vals = {}
    for n in ("q", "k", "v", "do"):
        t = torch.randn((S, H, d), generator=gen, device="cuda", dtype=torch.float32).bfloat16()
        vals[n] = t.view(torch.int16).cpu().numpy().view(np.uint16)
        del t
    torch.cuda.empty_cache()
    _sampled(oracle, w, rows_per_long=4, cols_per_long=0, seed=270, vals=vals, heads_per_row=3,
             wg_query_rows=wg_query_rows, window=128)


def test_shards_sum_to_unsharded_at_full_length():
    """GPU vs GPU at config 3's long length: O/LSE/dQ rows of each shard equal
    the unsharded rows bit for bit is not required (tiles differ), so compare
    within a few bf16 ulp; zero-padded partial dK/dV summed over the shards
    equal the unsharded dK/dV."""
    S, N, Hq, Hkv, d = 24576, 3, 8, 2, 128
    w = W.Workload("full", [S], [1], [0], Hq, Hkv, d, d ** -0.5, 606)
    full = run_library(w)
    dk_sum = np.zeros_like(full["dk"], dtype=np.float64)
    dv_sum = np.zeros_like(full["dv"], dtype=np.float64)
    L = S // N
    for r in range(N):
        b, e = r * L, (r + 1) * L
        vals = {"q": full["vals"]["q"][b:e], "do": full["vals"]["do"][b:e],
                "k": full["vals"]["k"][:e], "v": full["vals"]["v"][:e]}
        ws_ = W.Workload("shard", [S], [N], [r], Hq, Hkv, d, d ** -0.5, 606)
        sh = run_library(ws_, vals=vals)
        assert np.abs(sh["o"] - full["o"][b:e]).max() <= 2 * 2.0 ** -7 * max(1.0, np.abs(full["o"]).max())
        assert np.abs(sh["lse"] - full["lse"][:, b:e]).max() <= 1e-4
        assert np.abs(sh["dq"] - full["dq"][b:e]).max() <= 2 * 2.0 ** -7 * max(1.0, np.abs(full["dq"]).max())
        dk_sum[:e] += sh["dk"]
        dv_sum[:e] += sh["dv"]
        sh["plan"].destroy()
    for name, s_, f_ in (("dk", dk_sum, full["dk"]), ("dv", dv_sum, full["dv"])):
        err = np.abs(s_ - f_)
        tol = (N + 1) * 0.5 * bf16_ulp(np.maximum(np.abs(f_), 1.0)) + 1e-2
        assert (err <= tol).all(), (name, err.max())
    full["plan"].destroy()


# ---------------------------------------------------------------------------
# load-balanced cut: chunks r and 2N-1-r of 2N, two query segments on one prefix
# ---------------------------------------------------------------------------
TWO_CHUNK = {
    # name: (S, N, R, cut)
    "one_pair": ([1000], [4], [1], [1]),
    "first_and_last_rank": ([777, 777], [3, 3], [0, 2], [1, 1]),
    "degree_one_is_the_whole_sequence": ([300], [1], [0], [1]),
    "one_token_chunks": ([16, 130], [8, 1], [3, 0], [1, 0]),
    "mixed_with_local_and_contiguous": ([700, 2049, 129, 1030, 64], [1, 4, 1, 2, 1], [0, 2, 0, 1, 0], [0, 1, 0, 0, 0]),
    "ragged_everything": ([1001, 999, 515], [5, 7, 2], [4, 0, 1], [1, 1, 1]),
}


@pytest.mark.parametrize("name", sorted(TWO_CHUNK))
@pytest.mark.parametrize("heads,d", [((4, 2), 64), ((6, 2), 128)])
def test_two_chunk_cut(oracle, name, heads, d):
    S, N, R, Z = TWO_CHUNK[name]
    w = W.Workload(name, S, N, R, heads[0], heads[1], d, d ** -0.5, 900 + len(S) + d, shard_cut=Z)
    _exhaustive(oracle, w)


@pytest.mark.parametrize("bm,bn", [(64, 64), (64, 256), (256, 64), (128, 128), (0, 192)])
def test_two_chunk_cut_block_sizes(oracle, bm, bn):
    w = W.Workload("blocks2", [2100, 129, 1500], [3, 1, 2], [1, 0, 0], 4, 2, 128, 128 ** -0.5, 78,
                   shard_cut=[1, 0, 1])
    _exhaustive(oracle, w, bm, bn)


def test_two_chunk_cut_scaled_down_twin(oracle):
    """Structure of config 4 with the balanced cut, at a size the oracle covers."""
    w = W.scaled_shard_twin(seq_len=8192, degree=8, index=2)
    w.shard_cut = [1] + [0] * (len(w.seq_len) - 1)
    _exhaustive(oracle, w)


def test_two_chunk_cut_equals_its_two_slices_at_full_length():
    """GPU vs GPU at config 4's length (131,072 tokens, 8 ranks): the two segments of a
    two-chunk cut are the contiguous slices r and 2N-1-r of a 2N-way cut, which the
    sampled oracle tests above cover.  O / LSE / dQ run the same work items on the same
    rows, so they are equal bit for bit; dK / dV accumulate both chunks in fp32 and round
    once, where the separate runs round each partial sum, so those agree to rounding."""
    S, N, r, Hq, Hkv, d = 131072, 8, 2, 8, 2, 128
    wz = W.Workload("two_chunks", [S], [N], [r], Hq, Hkv, d, d ** -0.5, 707, shard_cut=[1])
    z = run_library(wz)
    c = S // (2 * N)
    la, lb = r * c, (2 * N - 1 - r) * c          # first rows of the two chunks
    assert z["plan"].total_q == 2 * c and z["plan"].total_k == lb + c and z["plan"].num_segments == 2
    dk = np.zeros_like(z["dk"], dtype=np.float64)
    dv = np.zeros_like(z["dv"], dtype=np.float64)
    for seg, (idx, first) in enumerate(((r, la), (2 * N - 1 - r, lb))):
        rows = slice(seg * c, (seg + 1) * c)
        vals = {"q": z["vals"]["q"][rows], "do": z["vals"]["do"][rows],
                "k": z["vals"]["k"][:first + c], "v": z["vals"]["v"][:first + c]}
        ws_ = W.Workload("slice", [S], [2 * N], [idx], Hq, Hkv, d, d ** -0.5, 707)
        one = run_library(ws_, vals=vals)
        assert np.array_equal(one["o"], z["o"][rows])
        assert np.array_equal(one["lse"], z["lse"][:, rows])
        assert np.array_equal(one["dq"], z["dq"][rows])
        dk[:first + c] += one["dk"]
        dv[:first + c] += one["dv"]
        one["plan"].destroy()
    for name, s_, f_ in (("dk", dk, z["dk"]), ("dv", dv, z["dv"])):
        err = np.abs(s_ - f_)
        tol = 1.5 * bf16_ulp(np.maximum(np.abs(f_), 1.0)) + 1e-2
        assert (err <= tol).all(), (name, err.max())
    # the pairs this rank attends are 1/N of the sequence's, up to rounding
    assert abs(z["plan"].attended_pairs - S * (S + 1) // 2 // N) <= 2 * S
    z["plan"].destroy()


# ---------------------------------------------------------------------------
# dK/dV head split: the query heads of a KV group shared out over several workgroups
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("heads,split", [((14, 2), 1), ((14, 2), 2), ((14, 2), 3), ((14, 2), 7),
                                         ((8, 2), 4), ((6, 6), 1), ((4, 1), 3)])
@pytest.mark.parametrize("d", [64, 128])
def test_head_split(oracle, heads, split, d):
    w = W.Workload("split", [700, 129, 2100, 64, 1500], [1, 1, 3, 1, 2], [0, 0, 1, 0, 1], heads[0], heads[1],
                   d, d ** -0.5, 88, shard_cut=[0, 0, 1, 0, 0])
    _exhaustive(oracle, w, head_split=split)


def test_head_split_is_chosen_from_the_work_list():
    from paper_2505_19609_amd import binding as B
    w2, w3 = W.config(2), W.config(3)
    p2 = B.skrull_attn_plan(w2.seq_len, w2.shard_degree, w2.shard_index, 14, 2, 64, 0.125)
    p3 = B.skrull_attn_plan(w3.seq_len, w3.shard_degree, w3.shard_index, 32, 8, 128, 0.1)
    base2 = (14 * p2.total_q * 8 + 255) // 256 * 256 + 256     # -D, LSE*log2e; the two work queues
    assert 1 < p2.head_split <= 7      # two KV heads and one long sequence: too few workgroups
    assert p2.bwd_workspace_bytes == base2 + 2 * p2.head_split * p2.total_k * 2 * 64 * 4
    assert p3.head_split == 1          # plenty of parallelism: the register-only path
    for bad in (-1, 8):
        with pytest.raises(B.SkrullError):
            B.skrull_attn_plan(w2.seq_len, w2.shard_degree, w2.shard_index, 14, 2, 64, 0.125, head_split=bad)
    p2.destroy(); p3.destroy()
    # the split follows r = longest chain / even share of the list over 256 compute units:
    # none up to r = 1, then the smallest divisor of the group size that is at least r
    for S, (hq, hkv, d), want in (([1024] * 16, (28, 4, 128), 1),   # r = 0.80
                                  ([4096] * 4, (28, 4, 128), 1),    # r = 0.94
                                  ([2048], (14, 2, 64), 7),         # r = 14
                                  ([4096], (32, 8, 128), 2),        # r = 1.88
                                  ([2048], (32, 8, 128), 4),        # r = 3.56
                                  ([8192] * 4, (14, 2, 64), 1)):    # r = 0.97
        p = B.skrull_attn_plan(S, [1] * len(S), [0] * len(S), hq, hkv, d, d ** -0.5, block_n=128)   # r is for 128-key items
        assert p.head_split == want, (S, hq, hkv, p.head_split)
        p.destroy()


@pytest.mark.parametrize("d,wg", [(64, 128), (64, 256), (128, 128), (128, 256)])
@pytest.mark.parametrize("jump", [12.0, 60.0, 100.0])
def test_forward_bound_follows_late_jumps(oracle, d, wg, jump):
    """The pipelined forward step takes its exponentials against the bound of the steps before and
    notices from their sum that the bound no longer holds.  Here a few keys deep inside long rows
    score `jump` (natural units after scaling) above everything before them for a set of query
    rows: 2^17 above the bound (sum far over its limit), 2^87, and 2^144 (the exponential
    overflows before the step is redone).  Other rows see the same keys with ordinary scores."""
    S = [2300, 1100]
    w = W.Workload(f"jump{jump}_{d}_{wg}", S, [1, 1], [0, 0], 4, 2, d, d ** -0.5, 606)
    from paper_2505_19609_amd import binding as B
    probe = B.skrull_attn_plan(S, [1, 1], [0, 0], 4, 2, d, w.softmax_scale)
    vals = W.make_values(w, probe.total_q, probe.total_k)
    probe.destroy()
    f = widen(vals)
    u = np.full(d, d ** -0.5, np.float32)                   # unit vector
    hot_keys = [1500, 1501, 1533, 2111, 2300 + 700]         # packed key rows (both sequences)
    hot_rows = list(range(1600, 1700, 7)) + [2200, 2299, 2300 + 900, 2300 + 1099]
    a = 8.0
    for j in hot_keys:
        f["k"][j, :, :] = (jump * d ** 0.5 / a) * u         # q.k * scale = jump for the hot rows
    for i in hot_rows:
        f["q"][i, :, :] = a * u
    vals = {n: W.f32_to_bf16_bits(x) for n, x in f.items()}
    out = run_library(w, vals=vals, wg_query_rows=wg)
    f = widen(out["vals"])
    desc = oracle.ranges(S, [1, 1], [0, 0])
    O, LSE = oracle.attention_fwd(f["q"], f["k"], f["v"], desc, w.softmax_scale)
    _report("O", out["o"], O, TOL_O)
    # LSE itself reaches `jump` here: a relative bound beside the absolute one (fp32 output)
    _report("LSE", out["lse"], LSE, TOL_O, rtol=1e-5)
    assert np.isfinite(out["dq"]).all() and np.isfinite(out["dk"]).all() and np.isfinite(out["dv"]).all()
    out["plan"].destroy()


@pytest.mark.parametrize("rows", [128, 256])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("bm", [0, 64])
def test_workgroup_shapes(oracle, rows, d, bm):
    """Both shapes of the forward and dQ kernels (4 wavefronts x 128 rows, fetching one tile
    ahead, and 8 x 256 with the deeper tile rings) on a micro-batch with one-tile, ragged
    and many-tile sequences and a distributed slice."""
    w = W.Workload(f"wg_rows{rows}_d{d}", [1, 63, 129, 700, 1411, 2600], [1, 1, 1, 1, 1, 2],
                   [0, 0, 0, 0, 0, 1], 4, 2, d, d ** -0.5, 77)
    _exhaustive(oracle, w, block_m=bm, wg_query_rows=rows)


@pytest.mark.parametrize("d", [64, 128])
def test_shapes_and_block_sizes_change_no_bit(d):
    """The workgroup shape of forward / dQ and the dK/dV block size (8 or 12 wavefronts at
    head_dim 64) only regroup the work: every result is bit-identical."""
    w = W.Workload("bitid", [1, 63, 129, 700, 1411, 2600, 5000], [1] * 6 + [2], [0] * 6 + [1], 4, 2, d, d ** -0.5, 77)
    base = run_library(w, wg_query_rows=128, head_split=1, block_n=128)
    for kw in (dict(wg_query_rows=256, block_n=128), dict(wg_query_rows=128, block_n=192),
               dict(wg_query_rows=256, block_n=256, block_m=64)):
        other = run_library(w, head_split=1, **kw)
        for n in ("o", "lse", "dq", "dk", "dv"):
            assert np.array_equal(base[n], other[n]), (kw, n)
        other["plan"].destroy()
    base["plan"].destroy()


def test_workgroup_shape_is_chosen_from_head_dim_and_amount_of_work():
    """wg_query_rows left open: 128 once the micro-batch holds enough work for the smaller
    workgroups to pay (head_dim 64: 24 blocks of 256 query rows x heads per compute unit, or 1.5e9
    attended (query, key, head) triples; head_dim 128: 16 such blocks and no sequence above 8,192
    tokens), else 256.  (256 compute units: 32 heads x 32,768 rows are 16 blocks per unit.)"""
    from paper_2505_19609_amd import binding as B
    for S, heads, d, want in (([8192] * 4, (32, 8), 128, 128), ([8193] + [8192] * 3, (32, 8), 128, 256),
                              ([8192, 100], (8, 2), 128, 256), ([1024] * 32, (28, 4), 128, 256),
                              ([1024] * 32, (64, 8), 128, 128), ([131072], (32, 8), 128, 256),
                              ([65536], (8, 2), 64, 128), ([1024] * 32, (64, 8), 64, 128),
                              ([1024] * 32, (32, 8), 64, 256), ([4096] * 8, (32, 8), 64, 128),
                              ([4096] * 8, (14, 2), 64, 256), ([8192] * 4, (14, 2), 64, 128),
                              ([300], (14, 2), 64, 256)):
        n = [8 if s > 100000 else 1 for s in S]
        plan = B.skrull_attn_plan(S, n, [0] * len(S), heads[0], heads[1], d, d ** -0.5)
        assert plan.info.wg_query_rows == want, (S, heads, d)
        plan.destroy()
        plan = B.skrull_attn_plan(S, n, [0] * len(S), heads[0], heads[1], d, d ** -0.5, wg_query_rows=384 - want)
        assert plan.info.wg_query_rows == 384 - want
        plan.destroy()


def test_dkv_block_is_chosen_from_head_dim_and_shape_of_the_work():
    """block_n left open: 192 (the 12-wavefront dK/dV shape) at head_dim 64 when a sequence
    of at least 8,192 tokens is present or the work list is short enough for the head
    split (longest chain above an even share of the 128-key items), else 128."""
    from paper_2505_19609_amd import binding as B
    for S, N, R, d, want in (([16384], [1], [0], 64, 192), ([8192] * 4, [1] * 4, [0] * 4, 64, 192),
                             ([1024] * 32, [1] * 32, [0] * 32, 64, 128), ([65536], [8], [7], 64, 192), ([8191], [1], [0], 64, 192), ([4096] * 8, [1] * 8, [0] * 8, 64, 128),
                             ([4096] * 2, [1] * 2, [0] * 2, 64, 192), ([3000] + [700] * 30, [1] * 31, [0] * 31, 64, 192),
                             ([65536], [8], [0], 64, 192), ([16384], [1], [0], 128, 128)):
        plan = B.skrull_attn_plan(S, N, R, 14, 2, d, d ** -0.5)
        assert plan.block_n == want, (S, N, R, d, plan.block_n)
        plan.destroy()
    plan = B.skrull_attn_plan([16384], [1], [0], 14, 2, 64, 0.125, block_n=128)
    assert plan.block_n == 128
    plan.destroy()
    # ... or when fewer, larger items still balance: five blocks of 192 key rows x KV heads per
    # compute unit (256 units), or a costliest 128-key item under 0.7 of the even share, and a
    # sequence of at least 384 tokens.  (Config 2's lengths with 8 KV heads: ratio 0.86, 760 items.)
    for S, heads, want in (([1024] * 32, (32, 8), 192), ([1024] * 26, (32, 8), 192),
                           ([256] * 128, (32, 8), 128), ([383] * 100, (16, 16), 128), ([384] * 100, (16, 16), 192),
                           ([1024] * 32, (32, 4), 192), (list(W.config(2).seq_len), (32, 8), 128),
                           (list(W.config(2).seq_len) * 2, (32, 8), 192)):
        plan = B.skrull_attn_plan(S, [1] * len(S), [0] * len(S), heads[0], heads[1], 64, 0.125)
        assert plan.block_n == want, (S[:2], len(S), heads, plan.block_n)
        plan.destroy()


def test_autograd_wrapper(oracle):
    """loss.backward() through the torch.autograd wrapper gives the library's gradients."""
    import torch
    from paper_2505_19609_amd import binding as B
    from paper_2505_19609_amd.autograd import skrull_attention
    from gpu_util import to_dev

    w = W.Workload("autograd", [300, 1000, 77], [1, 2, 1], [0, 1, 0], 4, 2, 64, 0.125, 321, shard_cut=[0, 1, 0])
    plan = B.skrull_attn_plan(w.seq_len, w.shard_degree, w.shard_index, 4, 2, 64, w.softmax_scale,
                              shard_cut=w.shard_cut)
    vals = W.make_values(w, plan.total_q, plan.total_k)
    dev = {n: to_dev(a) for n, a in vals.items()}
    q, k, v = (dev[n].clone().requires_grad_(True) for n in ("q", "k", "v"))
    o = skrull_attention(q, k, v, plan)
    (o.float() * dev["do"].float()).sum().backward()
    torch.cuda.synchronize()
    f = widen(vals)
    desc = oracle.ranges(w.seq_len, w.shard_degree, w.shard_index, w.shard_cut)
    O, _ = oracle.attention_fwd(f["q"], f["k"], f["v"], desc, w.softmax_scale)
    dQ, dK, dV, _ = oracle.attention_bwd(f["q"], f["k"], f["v"], f["do"], desc, w.softmax_scale)
    _report("O", o.detach().float().cpu().numpy(), O, TOL_O)
    _report("dQ", q.grad.float().cpu().numpy(), dQ, TOL_G)
    _report("dK", k.grad.float().cpu().numpy(), dK, TOL_G)
    _report("dV", v.grad.float().cpu().numpy(), dV, TOL_G)
    plan.destroy()


def test_mfma_ceiling_probe():
    """The measurement aid returns a rate between a third of and just above the nominal
    2.5 PFLOP/s (it is a pure MFMA loop at whatever clock the GPU holds)."""
    from paper_2505_19609_amd import binding as B
    rate = B.skrull_attn_mfma_ceiling()
    print(f"MFMA-only ceiling: {rate:.0f} TFLOP/s")
    assert 800.0 < rate < 2600.0

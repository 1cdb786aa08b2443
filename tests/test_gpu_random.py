"""Seeded random micro-batches (lengths, shard degrees and indices, both cuts, head
counts, head_dim, block sizes, head split, forward workgroup shape) against the fp64 oracle, exhaustively.
Every case is a valid problem; sizes are small enough for the oracle but span several
tiles, ragged tails, one-token chunks and every code path of the kernels."""
import numpy as np
import pytest

from paper_2505_19609_amd import workloads as W
from gpu_util import run_library, widen, bf16_ulp

pytestmark = pytest.mark.gpu

TOL_O, TOL_G = 2e-2, 5e-2


def _case(seed):
    rng = np.random.Generator(np.random.PCG64(10_000 + seed))
    K = int(rng.integers(1, 7))
    S, N, R, Z = [], [], [], []
    budget = 2600
    for _ in range(K):
        kind = rng.integers(0, 4)
        s = int(rng.integers(1, 40)) if kind == 0 else int(rng.integers(40, 700)) if kind < 3 else int(rng.integers(700, 1500))
        s = max(1, min(s, budget))
        z = int(rng.integers(0, 2))
        n = int(rng.integers(1, 9))
        n = max(1, min(n, s // (1 + z))) if s >= 1 + z else 1
        if n * (1 + z) > s:
            z = 0
            n = min(n, s)
        S.append(s); N.append(n); R.append(int(rng.integers(0, n))); Z.append(z)
        budget = max(1, budget - s)
    Hkv = int(rng.choice([1, 2, 3]))
    g = int(rng.choice([1, 2, 4, 7]))
    d = int(rng.choice([64, 128]))
    bm = int(rng.choice([0, 64, 128, 256]))
    bn = int(rng.choice([0, 64, 128, 256]))
    hs = int(rng.integers(0, g + 1))
    fr = int(rng.choice([0, 128, 256]))   # drawn last: the other parameters of a seed stay what they were
    if rng.integers(0, 4) == 0:
        bn = 192                           # (drawn after everything else, for the same reason)
    return S, N, R, Z, Hkv * g, Hkv, d, bm, bn, hs, fr


@pytest.mark.parametrize("seed", range(48))
def test_random_micro_batch(oracle, seed):
    S, N, R, Z, Hq, Hkv, d, bm, bn, hs, fr = _case(seed)
    print(f"seed {seed}: S={S} N={N} R={R} cut={Z} heads={Hq}/{Hkv} d={d} bm={bm} bn={bn} head_split={hs} "
          f"wg_query_rows={fr}", flush=True)
    w = W.Workload(f"rand{seed}", S, N, R, Hq, Hkv, d, d ** -0.5, 20_000 + seed, shard_cut=Z)
    out = run_library(w, bm, bn, head_split=hs, wg_query_rows=fr)
    f = widen(out["vals"])
    desc = oracle.ranges(S, N, R, Z)
    O, LSE = oracle.attention_fwd(f["q"], f["k"], f["v"], desc, w.softmax_scale)
    dQ, dK, dV, _ = oracle.attention_bwd(f["q"], f["k"], f["v"], f["do"], desc, w.softmax_scale)
    for name, got, ref, tol in (("O", out["o"], O, TOL_O), ("LSE", out["lse"], LSE, TOL_O),
                                ("dQ", out["dq"], dQ, TOL_G), ("dK", out["dk"], dK, TOL_G),
                                ("dV", out["dv"], dV, TOL_G)):
        assert np.isfinite(got).all(), name
        # max-abs tolerance; where the exact value is so large (|x| >= 16, e.g. dV of a one-token
        # sequence summed over 7 query heads) that half the spacing of the bf16 output exceeds
        # it, the correctly rounded output is the bound
        allowed = np.maximum(tol, 0.502 * bf16_ulp(ref))
        excess = float((np.abs(got - ref) - allowed).max()) if got.size else -1.0
        assert excess <= 0.0, (name, excess)
    out["plan"].destroy()

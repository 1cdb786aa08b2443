"""Pins of the GDS oracle (Sec. 4.3.2, Alg. 2) to things other than itself: hand-worked
examples, the constraints of the joint formulation (Sec. 4.2: every sequence in exactly
one micro-batch of one DP rank, at most C*N tokens per micro-batch), minimality of the
micro-batch count within the stride family, the interleave property, and the classical
guarantee of longest-processing-time bin packing against brute force."""
import itertools
import os
import random

import pytest

from oracle import dacp as OD
from oracle import gds as OG

GOLD = os.path.join(os.path.dirname(__file__), "golden", "gds_worked_examples.txt")
H, HKV = 4, 2


def _cases():
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        head, S, bins, mbs = [x.strip() for x in line.split("|")]
        ws, r, N, C = map(int, head.split())
        S = list(map(int, S.split()))
        bins = list(map(int, bins.split()))
        if mbs == "FAIL":
            want = None
        elif mbs == "-":
            want = []
        else:
            want = [[tuple(map(int, e.split(":"))) for e in mb.split()] for mb in mbs.split(";")]
        yield ws, r, N, C, S, bins, want


@pytest.mark.parametrize("case", list(_cases()), ids=lambda c: f"ws{c[0]}r{c[1]}N{c[2]}C{c[3]}")
def test_worked_examples(case):
    ws, r, N, C, S, bins, want = case
    assert OG.binpack(S, ws, H, HKV) == bins
    got = OG.gds_schedule(S, C, N, ws, r, H, HKV)
    if want is None:
        assert got is None
    else:
        assert got == (bins, want)


def _rand_batch(rng):
    K = rng.randint(1, 14)
    return [rng.choice([rng.randint(1, 6), rng.randint(1, 40)]) for _ in range(K)]


def test_constraints_and_minimality():
    rng = random.Random(5)
    n_multi = 0
    for _ in range(400):
        S = _rand_batch(rng)
        ws, N = rng.randint(1, 3), rng.randint(1, 4)
        C = rng.randint(max(1, max(S) // N), max(30, max(S)))
        per_rank = [OG.gds_schedule(S, C, N, ws, r, H, HKV) for r in range(ws)]
        if any(p is None for p in per_rank):
            # only a sequence longer than C*N may be unschedulable: one per micro-batch always works otherwise
            assert max(S) > C * N
            continue
        seen = [0] * len(S)
        for r, (bins, mbs) in enumerate(per_rank):
            assert bins == per_rank[0][0]
            tokens = sum(S[k] for k in range(len(S)) if bins[k] == r)
            for mb in mbs:
                ks = [k for k, _ in mb]
                assert all(bins[k] == r for k in ks)
                for k in ks:
                    seen[k] += 1
                assert sum(S[k] for k in ks) <= C * N                      # token constraint
                assert [S[k] for k in ks] == sorted(S[k] for k in ks)       # ascending inside
                # the decisions are those of DACP on this micro-batch, and they are feasible
                assert [t for _, t in mb] == OD.dacp_schedule([S[k] for k in ks], C, N, H, HKV)
                for j in range(N):
                    held = sum(S[k] if t == j else S[k] / N if t == -1 else 0 for k, t in mb)
                    assert held <= C + 1e-9
            m = len(mbs)
            if m:
                assert m >= -(-tokens // (C * N))                              # cannot be fewer
                sizes = [len(mb) for mb in mbs]
                if m < sum(sizes):  # stride cut: sizes differ by at most one, the m longest are apart
                    assert max(sizes) - min(sizes) <= 1
                longest = sorted((k for k in range(len(S)) if bins[k] == r), key=lambda k: (S[k], k))[-m:]
                where = {k: i for i, mb in enumerate(mbs) for k, _ in mb}
                assert len({where[k] for k in longest}) == min(m, len(longest))
                n_multi += m > 1
                # minimality inside the stride family: every smaller count breaks the token limit
                sub = sorted((k for k in range(len(S)) if bins[k] == r), key=lambda k: (S[k], k))
                for fewer in range(max(1, -(-tokens // (C * N))), m):
                    assert any(sum(S[k] for k in sub[j::fewer]) > C * N for j in range(fewer))
        assert seen == [1] * len(S)                                          # exactly once
    assert n_multi > 50


def test_binpack_lpt_bound_against_brute_force():
    rng = random.Random(11)
    for _ in range(150):
        ws = rng.randint(1, 3)
        S = [rng.randint(1, 60) for _ in range(rng.randint(1, 8))]
        cost = [OD.flops(s, H, HKV) for s in S]
        bins = OG.binpack(S, ws, H, HKV)
        assert all(0 <= b < ws for b in bins)
        got = max(sum(c for c, b in zip(cost, bins) if b == i) for i in range(ws))
        best = min(max(sum(c for c, b in zip(cost, a) if b == i) for i in range(ws))
                   for a in itertools.product(range(ws), repeat=len(S)))
        assert got * 3 * ws <= best * (4 * ws - 1)      # Graham's bound (4/3 - 1/(3 ws)) * OPT
        if len(S) <= ws:
            assert got == max(cost)                     # one sequence per bin is optimal


def test_binpack_special_cases():
    assert OG.binpack([7, 7, 7, 7], 2, H, HKV) == [0, 1, 0, 1]      # ties: caller's order, lowest bin
    assert OG.binpack([3, 9, 1], 1, H, HKV) == [0, 0, 0]
    # the cost is FLOPs(S), not S: with a large h the linear terms dominate and 3 x 10 tokens
    # balance one 30-token sequence; with h = 1 the quadratic term does not let them.
    assert OG.binpack([30, 10, 10, 10], 2, 4096, 1024) == [0, 1, 1, 1]
    big = OD.flops(30, 1, 1)
    assert big > 3 * OD.flops(10, 1, 1)

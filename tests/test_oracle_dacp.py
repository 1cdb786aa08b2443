"""Pins of the DACP oracle (oracle/dacp.py) against things other than itself:
hand-worked examples, the constraints Eq. 7 / Eq. 8 checked by brute force over
every (D, P) of tiny problems, textbook list scheduling when memory does not
bind, and the closed forms of FLOPs(S) the paper quotes (App. B.2)."""
import heapq
import itertools
import os
import random
from fractions import Fraction

import pytest

from oracle import dacp

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "dacp_worked_examples.txt")


def _examples():
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        a, b, c = [x.strip() for x in line.split("|")]
        N, C = map(int, a.split())
        S = list(map(int, b.split()))
        ret = None if c == "FAIL" else list(map(int, c.split()))
        yield N, C, S, ret


@pytest.mark.parametrize("N,C,S,want", list(_examples()))
def test_worked_examples(N, C, S, want):
    assert dacp.dacp_schedule(S, C, N, h=4, h_kv=2) == want


def _feasible(S, C, N, ret):
    """Eq. 7 and Eq. 8 written out: every sequence distributed or on exactly one
    rank; per rank, local tokens + S/N of every distributed sequence <= C."""
    if any(r != -1 and not (0 <= r < N) for r in ret):
        return False
    for j in range(N):
        used = sum(Fraction(s) for s, r in zip(S, ret) if r == j)
        used += sum(Fraction(s, N) for s, r in zip(S, ret) if r == -1)
        if used > C:
            return False
    return True


def _any_feasible(S, C, N):
    return any(_feasible(S, C, N, list(ret)) for ret in itertools.product(range(-1, N), repeat=len(S)))


def test_success_is_feasible_and_failure_only_when_tight_brute_force():
    rng = random.Random(7)
    n_ok = n_fail = n_infeasible = 0
    for _ in range(400):
        N = rng.choice([2, 3])
        K = rng.randint(1, 5)
        C = rng.randint(4, 14)
        S = [rng.randint(1, 16) for _ in range(K)]
        ret = dacp.dacp_schedule(S, C, N, h=8, h_kv=4)
        exists = _any_feasible(S, C, N)
        if ret is not None:
            n_ok += 1
            assert _feasible(S, C, N, ret), (S, C, N, ret)
            assert exists
        else:
            n_fail += 1
        if not exists:
            n_infeasible += 1
            assert ret is None, (S, C, N, ret)  # nothing can be scheduled where nothing fits
        # all-distributed is feasible exactly when sum(S)/N <= C; then some schedule must exist
        if sum(S) <= C * N:
            assert exists
    assert n_ok > 100 and n_fail > 20 and n_infeasible > 10  # the sample exercises every branch


def test_total_tokens_within_budget_always_schedules():
    """If sum(S) <= C*N the heuristic must succeed: sharding everything is feasible, and
    every roll-back moves the state towards it."""
    rng = random.Random(11)
    for _ in range(300):
        N = rng.choice([2, 4, 8])
        K = rng.randint(1, 12)
        S = [rng.randint(1, 50) for _ in range(K)]
        C = -(-sum(S) // N) + rng.randint(0, 3)
        ret = dacp.dacp_schedule(S, C, N, h=16, h_kv=4)
        assert ret is not None, (S, C, N)
        assert _feasible(S, C, N, ret)


def test_without_memory_pressure_it_is_list_scheduling():
    """C so large that the first branch always fits: Alg. 1 is then the textbook greedy
    'next job (ascending) to the least loaded machine', redone here with a heap."""
    rng = random.Random(3)
    for _ in range(100):
        N = rng.randint(1, 6)
        S = [rng.randint(1, 4000) for _ in range(rng.randint(1, 30))]
        ret = dacp.dacp_schedule(S, 10 ** 9, N, h=896, h_kv=128)
        heap = [(0, j) for j in range(N)]
        want = [None] * len(S)
        for k in sorted(range(len(S)), key=lambda k: (S[k], k)):
            load, j = heapq.heappop(heap)
            want[k] = j
            heapq.heappush(heap, (load + dacp.flops(S[k], 896, 128), j))
        assert ret == want


def test_order_of_the_input_does_not_matter():
    rng = random.Random(5)
    for _ in range(100):
        N = rng.choice([2, 4])
        S = [rng.randint(1, 40) for _ in range(rng.randint(2, 10))]
        C = rng.randint(max(S) // N + 1, sum(S))
        a = dacp.dacp_schedule(S, C, N, h=8, h_kv=2)
        perm = list(range(len(S)))
        rng.shuffle(perm)
        b = dacp.dacp_schedule([S[p] for p in perm], C, N, h=8, h_kv=2)
        if a is None:
            assert b is None
            continue
        # equal lengths may swap places; the multiset of (length, decision) is fixed
        assert sorted(zip(S, a)) == sorted(zip([S[p] for p in perm], b))


def test_flops_closed_forms_from_the_paper():
    # App. B.2, Qwen2.5-0.5B (h = 896, h_kv = 128): the quadratic term overtakes the linear
    # ones at S = (20 h^2 + 4 h h_kv) / (4 h) = 4608 ("approximately 4K"), and 32K costs
    # about 30x what 4K costs (34.35 by the formula).
    h, hkv = 896, 128
    lin = lambda S: 20 * h * h * S + 4 * h * hkv * S
    quad = lambda S: 4 * h * S * S
    assert lin(4608) == quad(4608)
    assert lin(4607) > quad(4607) and lin(4609) < quad(4609)
    assert dacp.flops(4608, h, hkv) == lin(4608) + quad(4608)
    r = dacp.flops(32768, h, hkv) / dacp.flops(4096, h, hkv)
    assert abs(r - 34.35) < 0.01
    # batch size multiplies every term
    assert dacp.flops(100, h, hkv, b=3) == 3 * dacp.flops(100, h, hkv)


def test_rank_batches_cover_every_sequence_once():
    S = [5, 100, 7, 64, 9]
    ret = [0, -1, 1, -1, 0]
    N = 2
    seen = []
    for j in range(N):
        seq, deg, idx, src = dacp.rank_batch(S, ret, N, j)
        for s, d, i, k in zip(seq, deg, idx, src):
            assert s == S[k]
            assert (d, i) == ((N, j) if ret[k] == -1 else (1, 0))
            seen.append((k, i if d > 1 else None))
    assert sorted(k for k, i in seen if i is None) == [0, 2, 4]
    assert sorted((k, i) for k, i in seen if i is not None) == [(1, 0), (1, 1), (3, 0), (3, 1)]

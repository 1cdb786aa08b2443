"""Pins for the oracle's integer part (descriptor + work lists).  CPU only."""
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_golden_shard_ranges(oracle):
    for line in open(os.path.join(GOLDEN, "shard_ranges.txt")):
        if line.startswith("#") or not line.strip():
            continue
        S, N, r, qb, ql, kv = (int(x) for x in line.split())
        d = oracle.ranges([S], [N], [r])
        assert (d["q_begin"][0], d["q_len"][0], d["kv_len"][0]) == (qb, ql, kv)


def test_unsharded_is_plain_cu_seqlens(oracle):
    S = [5, 1, 17, 300]
    d = oracle.ranges(S)
    assert list(d["cu_q"]) == [0, 5, 6, 23, 323]
    assert list(d["cu_k"]) == list(d["cu_q"])
    assert list(d["q_begin"]) == [0] * 4 and list(d["q_len"]) == S and list(d["kv_len"]) == S


@pytest.mark.parametrize("S,N", [(10, 3), (7, 7), (1000, 8), (13, 4), (131072, 8), (5, 2)])
def test_shards_tile_the_sequence(oracle, S, N):
    """Eq. 7 (completeness): the N slices are disjoint, ordered and cover [0, S);
    sizes differ by at most one and each shard's KV prefix ends where its queries do."""
    d = oracle.ranges([S] * N, [N] * N, list(range(N)))
    assert d["q_begin"][0] == 0
    for r in range(N):
        assert d["kv_len"][r] == d["q_begin"][r] + d["q_len"][r]
        if r + 1 < N:
            assert d["q_begin"][r + 1] == d["kv_len"][r]
    assert d["kv_len"][N - 1] == S and d["q_len"].sum() == S
    assert d["q_len"].max() - d["q_len"].min() <= 1
    assert d["total_q"] == S and d["total_k"] == int(d["kv_len"].sum())


def test_invalid_problems_rejected(oracle):
    for S, N, r in ([[0], [1], [0]], [[5], [0], [0]], [[5], [2], [2]], [[5], [2], [-1]], [[3], [4], [0]]):
        with pytest.raises(ValueError):
            oracle.ranges(S, N, r)


def _brute_pairs(desc):
    a = 0
    for k in range(desc["num_seqs"]):
        for i in range(desc["q_len"][k]):
            a += desc["q_begin"][k] + i + 1
    return a


def test_attended_pairs_brute_force(oracle):
    d = oracle.ranges([9, 40, 33, 1], [1, 4, 3, 1], [0, 2, 0, 0])
    assert oracle.attended_pairs(d) == _brute_pairs(d)
    full = oracle.ranges([64])
    assert oracle.attended_pairs(full) == 64 * 65 // 2


def test_shard_pair_ratio_is_2r_plus_1(oracle):
    """Eq. 4 charges every rank FLOPs/N; a contiguous causal cut really costs
    (2r+1)/N^2 of the sequence, i.e. index 7 of 8 does ~15x the pairs of index 0."""
    S, N = 131072, 8
    a = [oracle.attended_pairs(oracle.ranges([S], [N], [r])) for r in range(N)]
    assert sum(a) == S * (S + 1) // 2
    L = S // N
    for r in range(N):
        assert a[r] == ((2 * r + 1) * L * L + L) // 2
        assert a[r] == sum(range(r * L + 1, (r + 1) * L + 1))
    assert abs(a[7] / a[0] - 15.0) < 0.01


def _brute_tile_sets(desc, BM, BN):
    """All (seq, q_block, kv_block) tiles that contain at least one allowed pair."""
    tiles = set()
    for k in range(desc["num_seqs"]):
        for i in range(desc["q_len"][k]):
            p = desc["q_begin"][k] + i
            for nb in range(p // BN + 1):
                tiles.add((k, i // BM, nb))
    return tiles


@pytest.mark.parametrize("BM,BN", [(4, 4), (8, 4), (4, 8), (16, 16), (5, 3)])
def test_work_lists_cover_exactly_the_causal_tiles(oracle, BM, BN):
    S, N, r = [9, 40, 33, 1, 16, 17], [1, 4, 3, 1, 1, 2], [0, 2, 0, 0, 0, 1]
    d = oracle.ranges(S, N, r)
    tiles = _brute_tile_sets(d, BM, BN)
    f = oracle.fwd_items(d, BM, BN)
    g = oracle.dkv_items(d, BM, BN)
    # forward: item (k, m) visits kv blocks 0..n_kv-1
    ftiles = {(int(k), int(m), nb) for k, m, _, n in f for nb in range(n)}
    assert ftiles == tiles
    # dK/dV: item (k, n) is visited by q blocks m0..m0+n_q-1
    gtiles = {(int(k), m, int(n)) for k, n, m0, nq in g for m in range(m0, m0 + nq)}
    assert gtiles == tiles
    assert f[:, 3].sum() == g[:, 3].sum() == len(tiles)
    # q_row is the packed row of the block's first query
    for k, m, row, _ in f:
        assert row == d["cu_q"][k] + m * BM
    # one item per block, each exactly once
    assert len({(k, m) for k, m, _, _ in f}) == len(f) == sum(-(-int(q) // BM) for q in d["q_len"])
    assert len({(k, n) for k, n, _, _ in g}) == len(g) == sum(-(-int(q) // BN) for q in d["kv_len"])


def test_work_lists_sorted_stably(oracle):
    d = oracle.ranges([300, 64, 300, 1000, 17], [1, 1, 1, 4, 1], [0, 0, 0, 2, 0])
    for items in (oracle.fwd_items(d, 32, 32), oracle.dkv_items(d, 32, 32)):
        cost = items[:, 3]
        assert np.all(cost[:-1] >= cost[1:])
        # ties keep (seq, block) ascending
        for a, b in zip(items[:-1], items[1:]):
            if a[3] == b[3]:
                assert (a[0], a[1]) < (b[0], b[1])


def test_fwd_cost_closed_form(oracle):
    """Unsharded sequence of length L with BM = BN = B: block m sees m+1 key blocks."""
    d = oracle.ranges([1000])
    f = oracle.fwd_items(d, 128, 128)
    assert sorted(f[:, 3].tolist()) == list(range(1, 9))
    g = oracle.dkv_items(d, 128, 128)
    assert sorted(g[:, 3].tolist()) == list(range(1, 9))
    assert list(g[:, 2] + g[:, 3]) == [8] * 8

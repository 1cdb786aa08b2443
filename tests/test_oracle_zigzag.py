"""Pins of the oracle's load-balanced two-chunk cut (chunks r and 2N-1-r of 2N) to
things other than itself: the unsharded definition of the same sequence (a rank's O /
LSE / dQ rows are the whole sequence's rows at the same positions; the ranks' partial
dK / dV add up to the whole sequence's), the partition of the positions, the balance
the cut exists for (every rank attends S(S+1)/2N pairs up to rounding), the degenerate
case N = 1, and brute-force tile counting for the dK/dV work list."""
import numpy as np
import pytest

import oracle
from paper_2505_19609_amd import workloads as W


def _vals(T, Hq, Hkv, d, seed):
    w = W.Workload("z", [T], [1], [0], Hq, Hkv, d, d ** -0.5, seed)
    return {n: W.bf16_bits_to_f32(a) for n, a in W.make_values(w, T, T).items()}


@pytest.mark.parametrize("S,N", [(97, 3), (128, 4), (61, 1), (40, 5)])
def test_chunks_partition_positions_and_balance_pairs(S, N):
    seen = np.zeros(S, np.int32)
    pairs = []
    for r in range(N):
        d = oracle.ranges([S], [N], [r], [1])
        assert d["num_seqs"] == 2 and list(d["shares_kv"]) == [0, 1]
        a, b = (range(d["q_begin"][s], d["q_begin"][s] + d["q_len"][s]) for s in (0, 1))
        assert a.stop <= b.start                     # early chunk first
        for p in list(a) + list(b):
            seen[p] += 1
        assert d["cu_k"][0] == d["cu_k"][1] == 0 and d["total_k"] == b.stop == d["kv_len"][1]
        assert d["kv_len"][0] == a.stop and d["cu_q"][1] == len(a) and d["total_q"] == len(a) + len(b)
        assert abs(len(a) + len(b) - S / N) < 2      # Eq. 8: S/N tokens per rank
        pairs.append(oracle.attended_pairs(d))
    assert (seen == 1).all()
    assert sum(pairs) == S * (S + 1) // 2
    # balance: every rank within one row's worth of pairs per chunk boundary of the mean
    assert max(pairs) - min(pairs) <= 4 * S
    if N > 1:   # the contiguous cut is far from it
        contiguous = [oracle.attended_pairs(oracle.ranges([S], [N], [r])) for r in range(N)]
        assert max(contiguous) - min(contiguous) > max(pairs) - min(pairs)


@pytest.mark.parametrize("S,N,heads,d", [(75, 3, (4, 2), 16), (64, 2, (2, 1), 32), (33, 1, (2, 2), 16)])
def test_ranks_reassemble_to_the_unsharded_sequence(S, N, heads, d):
    Hq, Hkv = heads
    f = _vals(S, Hq, Hkv, d, 77)
    full = oracle.ranges([S])
    scale = d ** -0.5
    O, LSE = oracle.attention_fwd(f["q"], f["k"], f["v"], full, scale)
    dQ, dK, dV, _ = oracle.attention_bwd(f["q"], f["k"], f["v"], f["do"], full, scale)
    dk_sum, dv_sum = np.zeros_like(dK), np.zeros_like(dV)
    for r in range(N):
        z = oracle.ranges([S], [N], [r], [1])
        pos = np.concatenate([np.arange(z["q_begin"][s], z["q_begin"][s] + z["q_len"][s]) for s in (0, 1)])
        e = z["total_k"]
        o, lse = oracle.attention_fwd(f["q"][pos], f["k"][:e], f["v"][:e], z, scale)
        dq, dk, dv, _ = oracle.attention_bwd(f["q"][pos], f["k"][:e], f["v"][:e], f["do"][pos], z, scale)
        np.testing.assert_allclose(o, O[pos], rtol=0, atol=1e-12)
        np.testing.assert_allclose(lse, LSE[:, pos], rtol=0, atol=1e-12)
        np.testing.assert_allclose(dq, dQ[pos], rtol=0, atol=1e-11)
        dk_sum[:e] += dk
        dv_sum[:e] += dv
    np.testing.assert_allclose(dk_sum, dK, rtol=0, atol=1e-10)
    np.testing.assert_allclose(dv_sum, dV, rtol=0, atol=1e-10)


def test_mixed_micro_batch_segments_and_offsets():
    # local, two-chunk shard, contiguous shard, local: segment arrays and packed offsets
    d = oracle.ranges([10, 40, 33, 5], [1, 4, 3, 1], [0, 1, 2, 0], [0, 1, 0, 0])
    assert d["num_seqs"] == 5
    assert list(d["q_begin"]) == [0, 5, 30, 22, 0]       # 40/8 = 5 per chunk: chunks 1 and 6
    assert list(d["q_len"]) == [10, 5, 5, 11, 5]
    assert list(d["kv_len"]) == [10, 10, 35, 33, 5]
    assert list(d["shares_kv"]) == [0, 0, 1, 0, 0]
    assert list(d["cu_q"]) == [0, 10, 15, 20, 31, 36]
    assert list(d["cu_k"]) == [0, 10, 10, 45, 78, 83]
    with pytest.raises(ValueError):
        oracle.ranges([7], [4], [0], [1])                # 8 chunks need 8 tokens
    with pytest.raises(ValueError):
        oracle.ranges([70], [4], [0], [2])


@pytest.mark.parametrize("BM,BN", [(4, 4), (8, 4), (4, 16)])
def test_dkv_items_of_a_shared_prefix_by_brute_force(BM, BN):
    d = oracle.ranges([50, 9], [3, 1], [1, 0], [1, 0])   # chunks 1 and 4 of 6
    items = oracle.dkv_items(d, BM, BN)
    # one item per key block of each PREFIX, owned by its last segment
    assert sorted((k, b) for k, b, _, _ in items) == \
        [(1, b) for b in range(-(-d["kv_len"][1] // BN))] + [(2, b) for b in range(-(-9 // BN))]
    for k, b, m0, cost in items:
        segs = [k - 1, k] if d["shares_kv"][k] else [k]
        blocks = set()
        for s in segs:
            for i in range(d["q_len"][s]):
                if d["q_begin"][s] + i >= b * BN:          # this row sees the block's first key
                    blocks.add((s, i // BM))
        assert cost == len(blocks)
        assert m0 == min(m for s, m in blocks if s == k)
    assert list(items[:, 3]) == sorted(items[:, 3], reverse=True)

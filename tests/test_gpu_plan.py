"""Exact integer parity of the device-built descriptor and work lists with the oracle."""
import numpy as np
import pytest

from paper_2505_19609_amd import workloads as W

pytestmark = pytest.mark.gpu

CASES = {
    "one_token": ([1], [1], [0]),
    "block_edges": ([63, 64, 65, 127, 128, 129, 255, 256, 257], [1] * 9, [0] * 9),
    "ragged_shards": ([1000, 999, 7, 130, 4096], [3, 7, 7, 2, 5], [1, 6, 0, 1, 4]),
    "many_short": (list(range(1, 400)), [1] * 399, [0] * 399),
}


def _check(oracle, S, N, R, Hq, Hkv, d, bm, bn, cut=None):
    from paper_2505_19609_amd import binding as B
    plan = B.skrull_attn_plan(S, N, R, Hq, Hkv, d, 0.1, bm, bn, shard_cut=cut)
    desc = oracle.ranges(S, N, R, cut)
    assert plan.num_seqs == len(S) and plan.num_segments == desc["num_seqs"]
    BM, BN = plan.block_m, plan.block_n
    assert BM == (bm or 256) and (BN == bn if bn else BN in (128, 192))   # 0: the library's choice
    assert plan.total_q == desc["total_q"] and plan.total_k == desc["total_k"]
    assert plan.attended_pairs == oracle.attended_pairs(desc)
    assert plan.useful_flops_fwd == 4 * plan.attended_pairs * d * Hq
    assert plan.useful_flops_bwd == 10 * plan.attended_pairs * d * Hq
    assert plan.bwd_workspace_bytes >= 4 * Hq * plan.total_q
    for which, name in ((B.ARRAY_CU_Q, "cu_q"), (B.ARRAY_CU_K, "cu_k"), (B.ARRAY_Q_BEGIN, "q_begin"),
                        (B.ARRAY_Q_LEN, "q_len"), (B.ARRAY_KV_LEN, "kv_len"),
                        (B.ARRAY_SHARES_KV, "shares_kv")):
        assert np.array_equal(B.skrull_attn_plan_export(plan, which), desc[name]), name
    assert np.array_equal(B.skrull_attn_plan_export(plan, B.ARRAY_FWD_ITEMS), oracle.fwd_items(desc, BM, BN))
    assert np.array_equal(B.skrull_attn_plan_export(plan, B.ARRAY_DKV_ITEMS), oracle.dkv_items(desc, BM, BN))
    plan.destroy()


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("bm,bn", [(0, 0), (64, 256), (256, 64), (128, 192)])
def test_plan_matches_oracle_on_benchmark_configs(oracle, n, bm, bn):
    w = W.config(n)
    _check(oracle, w.seq_len, w.shard_degree, w.shard_index, w.num_q_heads, w.num_kv_heads, w.head_dim, bm, bn)
    if n == 4:
        w0 = W.config(4, shard_index=0)
        _check(oracle, w0.seq_len, w0.shard_degree, w0.shard_index, 32, 8, 128, bm, bn)


@pytest.mark.parametrize("name", sorted(CASES))
@pytest.mark.parametrize("bm,bn", [(0, 0), (64, 64), (128, 256), (256, 192)])
def test_plan_matches_oracle_on_edge_cases(oracle, name, bm, bn):
    S, N, R = CASES[name]
    _check(oracle, S, N, R, 4, 2, 64, bm, bn)


TWO_CHUNK_CASES = {
    "one_pair": ([1000], [4], [1], [1]),
    "every_rank": ([4099] * 5, [5] * 5, [0, 1, 2, 3, 4], [1] * 5),
    "one_token_chunks": ([16, 130, 6], [8, 1, 3], [3, 0, 2], [1, 0, 1]),
    "mixed": ([700, 2049, 129, 1030, 64, 40000], [1, 4, 1, 2, 1, 8], [0, 2, 0, 1, 0, 5], [0, 1, 0, 0, 1, 1]),
}


@pytest.mark.parametrize("name", sorted(TWO_CHUNK_CASES))
@pytest.mark.parametrize("bm,bn", [(0, 0), (64, 64), (128, 256), (256, 64), (64, 192)])
def test_plan_matches_oracle_with_two_chunk_cuts(oracle, name, bm, bn):
    S, N, R, Z = TWO_CHUNK_CASES[name]
    _check(oracle, S, N, R, 4, 2, 64, bm, bn, cut=Z)


def test_plan_many_two_chunk_sequences(oracle):
    rng = np.random.Generator(np.random.PCG64(8))
    S = rng.integers(2, 600, size=1500).tolist()
    Z = rng.integers(0, 2, size=1500).tolist()
    N = [int(min(s // (1 + z), n)) for s, z, n in zip(S, Z, rng.integers(1, 6, size=1500))]
    R = [int(rng.integers(0, n)) for n in N]
    _check(oracle, S, N, R, 8, 8, 128, 0, 0, cut=Z)


def test_plan_rejects_bad_cuts():
    from paper_2505_19609_amd import binding as B
    for S, N, R, Z in (([7], [4], [0], [1]), ([70], [4], [0], [2]), ([70], [4], [0], [-1])):
        with pytest.raises(B.SkrullError) as e:
            B.skrull_attn_plan(S, N, R, 4, 2, 64, 0.1, shard_cut=Z)
        assert e.value.code == B.SKRULL_EINVAL


def test_plan_large_sequence_count(oracle):
    rng = np.random.Generator(np.random.PCG64(7))
    S = rng.integers(1, 300, size=3000).tolist()
    N = [int(min(s, n)) for s, n in zip(S, rng.integers(1, 5, size=3000))]
    R = [int(rng.integers(0, n)) for n in N]
    _check(oracle, S, N, R, 8, 8, 128, 0, 0)


def test_plan_rejects_oversized_total():
    from paper_2505_19609_amd import binding as B
    with pytest.raises(B.SkrullError) as e:
        B.skrull_attn_plan([2 ** 30, 2 ** 30, 2 ** 30], [1] * 3, [0] * 3, 8, 8, 128, 0.1)
    assert e.value.code == B.SKRULL_EINVAL


@pytest.mark.timeout(300)
@pytest.mark.parametrize("longest,passes", [(250, 1), (10_000, 2), (4_200_000, 3)])
def test_plan_long_lists_are_radix_sorted(oracle, longest, passes):
    """More than 2,048 work items per list (here 18,000 and more): the plan sorts by stable radix passes (one, two or
    three 8-bit digits, depending on the largest possible cost) instead of by rank counting;
    the layout stays exactly the oracle's."""
    rng = np.random.Generator(np.random.PCG64(70 + passes))
    S = rng.integers(1, 250, size=18_000).tolist()
    if longest > 250:
        S.insert(7, longest)
    N = [int(min(s, n)) for s, n in zip(S, rng.integers(1, 4, size=len(S)))]
    R = [int(rng.integers(0, n)) for n in N]
    if longest > 250:
        N[7], R[7] = 1, 0
    assert 2 * (longest // 64 + 2) >= 256 ** (passes - 1) and 2 * (longest // 64 + 2) < 256 ** passes
    _check(oracle, S, N, R, 1, 1, 64, 64, 64)

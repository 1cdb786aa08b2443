"""The synthetic inputs: the five benchmark micro-batches have the shapes their
descriptions give, the Table 1 length generator reproduces the paper's shares, the
bf16 conversion rounds to nearest even, and bench.py refuses more than one GPU."""
import os
import subprocess
import sys

import numpy as np
import pytest

from paper_2505_19609_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_config1_is_the_literal_tiny_batch():
    w = W.config(1)
    assert w.seq_len == [37, 128, 256, 511] and sum(w.seq_len) == 932
    assert (w.num_q_heads, w.num_kv_heads, w.head_dim) == (4, 4, 64)
    assert w.shard_degree == [1] * 4 and w.q_prescale == 0.125 and w.value_seed == 0


@pytest.mark.parametrize("n, heads, budget, clip", [
    (2, (14, 2, 64), 16384, (16, 8192)),
    (3, (32, 8, 128), 32768, (32, 4096)),
])
def test_unsharded_configs_fill_their_token_budget(n, heads, budget, clip):
    w = W.config(n)
    assert (w.num_q_heads, w.num_kv_heads, w.head_dim) == heads
    assert sum(w.seq_len) == budget and set(w.shard_degree) == {1}
    assert w.softmax_scale == pytest.approx(heads[2] ** -0.5)
    short = w.seq_len[1:] if n == 3 else w.seq_len
    assert min(short) >= clip[0] and max(short) <= clip[1]
    if n == 3:   # one long sequence, the rest short: 99 % of the sequences would need > 100 of them,
        # a 32,768-token budget holds fewer; the composition (24,576 + 8,192 short tokens) is what is kept
        assert w.seq_len[0] == 24576 and sum(short) == 8192


def test_config4_is_one_shard_of_a_131072_token_sequence_plus_short_ones():
    for r in (7, 0):
        w = W.config(4, shard_index=r)
        assert w.seq_len[0] == 131072 and w.shard_degree[0] == 8 and w.shard_index[0] == r
        assert set(w.shard_degree[1:]) == {1} and sum(w.seq_len[1:]) == 8192
        assert min(w.seq_len[1:]) >= 64 and max(w.seq_len[1:]) <= 4096
        assert (w.num_q_heads, w.num_kv_heads, w.head_dim) == (32, 8, 128)
    assert W.config(4).shard_index[0] == 7   # the default is the last, heaviest slice


def test_config5_is_bimodal_plus_a_quarter_of_a_65536_token_sequence():
    w = W.config(5)
    assert (w.num_q_heads, w.num_kv_heads, w.head_dim) == (28, 4, 128)
    assert (w.seq_len[0], w.shard_degree[0], w.shard_index[0]) == (65536, 4, 3)
    rest = w.seq_len[1:]
    longs = [s for s in rest if s >= 16384]
    assert sum(rest) == 65536 and set(w.shard_degree[1:]) == {1}
    assert all(16384 <= s <= 49152 for s in longs)
    assert sum(longs) >= 0.4 * 65536 and sum(longs) - longs[-1] < 0.4 * 65536   # just past 40 % of the tokens
    assert all(32 <= s <= 8192 for s in rest if s < 16384)


def test_configs_are_reproducible():
    for n in range(1, 6):
        assert W.config(n).seq_len == W.config(n).seq_len
    a = W.make_values(W.config(1), 932, 932)
    b = W.make_values(W.config(1), 932, 932)
    assert all((a[k] == b[k]).all() for k in a)
    q = W.bf16_bits_to_f32(a["q"])
    assert abs(q.std() - 0.125) < 0.002 and abs(W.bf16_bits_to_f32(a["k"]).std() - 1.0) < 0.01


@pytest.mark.parametrize("dataset", sorted(W.TABLE1))
def test_table1_shares(dataset):
    """Paper Table 1: the shares of sequences below 1K / 4K / 8K / 32K / 128K tokens."""
    rng = np.random.Generator(np.random.PCG64(5))
    S = np.array(W.table1_lengths(rng, dataset, count=200_000))
    cdf, cap = W.TABLE1[dataset]
    for edge, share in zip(W.TABLE1_EDGES[1:], cdf):
        assert abs((S < edge).mean() - share) < 0.004, (edge, share)
    assert S.min() >= W.TABLE1_EDGES[0] and S.max() <= cap


def test_table1_budget_and_cap():
    rng = np.random.Generator(np.random.PCG64(6))
    for _ in range(50):
        S = W.table1_lengths(rng, "chatqa2_long_sft", budget=100_000, longest=40_000)
        assert 0 < sum(S) <= 100_000 and max(S) <= 40_000
    assert len(W.table1_lengths(rng, "wikipedia", count=17)) == 17


def test_bf16_rounding_is_to_nearest_even():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -2.5, 0.0], np.float32)
    back = W.bf16_bits_to_f32(W.f32_to_bf16_bits(x))
    # ties go to the even significand: 1 + 2^-8 -> 1, 1 + 3*2^-8 -> 1 + 2^-6; just above a tie rounds up
    assert back.tolist() == [1.0, 1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -2.5, 0.0]


def test_model_shapes_match_their_head_counts():
    for name, (h, hkv, hq, hk, d) in W.MODEL_SHAPES.items():
        assert h == hq * d and hkv == hk * d, name


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "--gpus 1" in r.stderr and not r.stdout.strip()

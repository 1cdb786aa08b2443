"""The library's GDS scheduler (host code behind the C ABI) against the oracle, decision
for decision, on global batches drawn from the paper's length mixes (Table 1) at the
paper's settings (BatchSize 64 per DP rank, DP 4, CP 8, BucketSize 26K / 13K; Sec. 5) and
on adversarial tiny ones.  No GPU needed."""
import os
import random

import numpy as np
import pytest

from oracle import gds as OG
from paper_2505_19609_amd import workloads as W


@pytest.fixture(scope="module")
def B():
    from paper_2505_19609_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2505_19609_amd import build
        build.build_library()
    return binding


def _compare(B, S, C, N, ws, h, hkv):
    outcomes = []
    for r in range(ws):
        want = OG.gds_schedule(S, C, N, ws, r, h, hkv)
        try:
            bins, mb, ret, m = B.skrull_gds_schedule(S, C, N, ws, r, h, hkv)
        except B.SkrullError as e:
            assert e.code == B.SKRULL_ESCHED
            assert want is None, (S, C, N, ws, r)
            outcomes.append(None)
            continue
        assert want is not None, (S, C, N, ws, r)
        wbins, wmbs = want
        assert list(bins) == wbins == list(B.skrull_gds_binpack(S, ws, h, hkv))
        assert m == len(wmbs)
        for j, wmb in enumerate(wmbs):
            members = B.skrull_gds_micro_batch(S, mb, j)
            assert [(int(k), int(ret[k])) for k in members] == wmb
        others = [k for k in range(len(S)) if wbins[k] != r]
        assert all(mb[k] == -1 and ret[k] == -2 for k in others)
        outcomes.append(m)
    return outcomes


def test_tiny_batches_match_oracle(B):
    rng = random.Random(21)
    fails = multi = 0
    for _ in range(300):
        S = [rng.choice([rng.randint(1, 6), rng.randint(1, 40)]) for _ in range(rng.randint(1, 14))]
        ws, N = rng.randint(1, 3), rng.randint(1, 4)
        C = rng.randint(max(1, max(S) // (2 * N)), max(30, max(S)))
        out = _compare(B, S, C, N, ws, *rng.choice([(4, 2), (896, 128)]))
        fails += any(o is None for o in out)
        multi += any(o is not None and o > 1 for o in out)
    assert fails > 5 and multi > 50


@pytest.mark.parametrize("dataset,model,C", [("wikipedia", "qwen2.5-0.5b", 26 * 1024),
                                             ("chatqa2_long_sft", "qwen2.5-0.5b", 26 * 1024),
                                             ("chatqa2_long_sft", "qwen2.5-7b", 13 * 1024),
                                             ("lmsyschat1m", "qwen2.5-7b", 13 * 1024)])
def test_paper_settings_match_oracle(B, dataset, model, C):
    h, hkv = W.MODEL_SHAPES[model][:2]
    for seed in range(3):
        rng = np.random.Generator(np.random.PCG64(seed))
        S = W.table1_lengths(rng, dataset, count=4 * 64, longest=C * 8)
        out = _compare(B, S, C, 8, 4, h, hkv)
        assert all(o is not None and o >= 1 for o in out)


def test_argument_errors(B):
    ok = dict(seq_len=[5, 6, 7], bucket_size=10, cp_degree=2, dp_world_size=2, dp_rank=0, hidden=8, hidden_kv=2)
    for bad in (dict(seq_len=[5, 0]), dict(seq_len=[]), dict(bucket_size=0), dict(cp_degree=0),
                dict(dp_world_size=0), dict(dp_rank=2), dict(dp_rank=-1), dict(hidden=0), dict(batch=0)):
        with pytest.raises(B.SkrullError) as e:
            B.skrull_gds_schedule(**{**ok, **bad})
        assert e.value.code == B.SKRULL_EINVAL
    with pytest.raises(B.SkrullError) as e:
        B.skrull_gds_binpack([3, 4], 0, 8, 2)
    assert e.value.code == B.SKRULL_EINVAL
    with pytest.raises(B.SkrullError) as e:
        B.skrull_gds_micro_batch([3, 4], [0, 0], -1)
    assert e.value.code == B.SKRULL_EINVAL
    with pytest.raises(B.SkrullError) as e:   # 50 tokens can never fit C*N = 20
        B.skrull_gds_schedule([50, 3], 10, 2, 1, 0, 8, 2)
    assert e.value.code == B.SKRULL_ESCHED

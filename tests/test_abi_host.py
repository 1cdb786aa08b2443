"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every declared symbol, and rejects invalid problems before touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2505_19609_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2505_19609_amd import build
        build.build_library()
    return binding


def test_library_exports_every_declared_symbol(B):
    inc = os.path.join(ROOT, "include")
    header = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    declared = set(re.findall(r"\b(skrull_(?:attn|dacp|gds)_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTED_SYMBOLS)
    L = B.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_struct_layouts_match_header(B):
    # 4+pad, 3 pointers, 3 ints, float, 2 ints, 1 pointer, 2 ints
    assert ctypes.sizeof(B.Problem) == 72
    assert ctypes.sizeof(B.PlanInfo) == 10 * 4 + 4 * 8 + 4 * 4


def test_strerror(B):
    assert B.skrull_attn_strerror(0) == "ok"
    assert "invalid" in B.skrull_attn_strerror(B.SKRULL_EINVAL)
    assert "gfx950" in B.skrull_attn_strerror(B.SKRULL_EUNSUPPORTED)
    assert "unknown" in B.skrull_attn_strerror(-99)


@pytest.mark.parametrize("kw", [
    dict(seq_len=[]), dict(seq_len=[0]), dict(shard_degree=[0]), dict(shard_index=[1]),
    dict(shard_index=[-1]), dict(seq_len=[3], shard_degree=[4]), dict(num_q_heads=6, num_kv_heads=4),
    dict(num_q_heads=0), dict(num_kv_heads=0), dict(head_dim=96), dict(softmax_scale=0.0),
    dict(softmax_scale=float("nan")), dict(softmax_scale=float("inf")), dict(block_m=96),
    dict(block_m=32), dict(block_n=2048), dict(block_m=512), dict(wg_query_rows=64), dict(wg_query_rows=-1),
    # 32-bit tile offsets: (S + 256) * Hkv * d * 2 and (chunk + 256) * Hq * d * 2 must stay below 2^32
    dict(seq_len=[2_096_896], num_q_heads=8, num_kv_heads=8, head_dim=128, shard_degree=[8], shard_index=[0]),
    dict(seq_len=[524_032], num_q_heads=32, num_kv_heads=8, head_dim=128),
])
def test_invalid_problems_return_einval_without_a_device(B, kw):
    args = dict(seq_len=[10], shard_degree=[1], shard_index=[0], num_q_heads=4, num_kv_heads=2,
                head_dim=64, softmax_scale=0.125, block_m=0, block_n=0)
    args.update(kw)
    with pytest.raises(B.SkrullError) as e:
        B.skrull_attn_plan(raw_stream=0, **args)
    assert e.value.code == B.SKRULL_EINVAL


def test_longest_addressable_sequences_pass_the_entry_checks(B):
    """One row under the 32-bit offset limits: the checks that need no device pass
    (the call then stops at the missing GPU, or succeeds where there is one)."""
    import torch
    for kw in (dict(seq_len=[2_096_895], num_q_heads=8, num_kv_heads=8, head_dim=128, shard_degree=[8], shard_index=[0]),
               dict(seq_len=[524_031], num_q_heads=32, num_kv_heads=8, head_dim=128, shard_degree=[1], shard_index=[0])):
        args = dict(softmax_scale=0.125, block_m=0, block_n=0)
        args.update(kw)
        if torch.cuda.is_available():
            B.skrull_attn_plan(**args).destroy()
        else:
            with pytest.raises(B.SkrullError) as e:
                B.skrull_attn_plan(raw_stream=0, **args)
            assert e.value.code == B.SKRULL_EUNSUPPORTED


def test_null_arguments(B):
    L = B.lib()
    assert L.skrull_attn_plan(None, None, None) == B.SKRULL_EINVAL
    assert L.skrull_attn_plan_info(None, None) == B.SKRULL_EINVAL
    assert L.skrull_attn_plan_export(None, 0, None, 0) == B.SKRULL_EINVAL
    assert L.skrull_attn_fwd(None, None, None, None, None, None, None) == B.SKRULL_EINVAL
    assert L.skrull_attn_bwd(*([None] * 11), 0, None) == B.SKRULL_EINVAL
    assert L.skrull_attn_bwd_static(*([None] * 11)) == B.SKRULL_EINVAL
    assert L.skrull_attn_trace_layout(None, None, None) == B.SKRULL_EINVAL
    assert L.skrull_attn_trace(None, 0) == B.SKRULL_OK            # "off" needs no device
    assert L.skrull_attn_profile_read(None) == B.SKRULL_EINVAL
    import ctypes as C
    assert L.skrull_attn_profile_read((C.c_float * 4)()) == B.SKRULL_EINVAL   # this thread never enabled it
    L.skrull_attn_plan_destroy(None)


def test_valid_problem_without_gpu_is_unsupported_not_a_crash(B):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(B.SkrullError) as e:
        B.skrull_attn_plan([10], [1], [0], 4, 2, 64, 0.125, raw_stream=0)
    assert e.value.code == B.SKRULL_EUNSUPPORTED

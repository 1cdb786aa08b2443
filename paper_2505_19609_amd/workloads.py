"""Seeded synthetic micro-batches: sequence-length mixes and bf16 token values.

This module serves both the HIP library's tests/benchmark and the CPU oracle's
tests.  It holds none of the method's arithmetic: it only draws sequence
lengths and i.i.d. values and rounds them to bf16, so that both sides can be
fed the same bytes.

The length mixes stand in for the corpora the paper trains on (its Table 1:
a long-tail mix where ~88 % of sequences are under 1K tokens and ~99 % under
4K, and a bimodal mix with 40 % long sequences; Sec. 1 quotes the Llama-3 and
Qwen2.5-Turbo recipes).  Only the length distribution matters to attention
cost, so values are N(0,1).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass
class Workload:
    name: str
    seq_len: list          # full (unsharded) length S_k of every sequence
    shard_degree: list     # 1 = local / whole, N > 1 = distributed over N ranks
    shard_index: list      # which 1/N slice this GPU holds
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    softmax_scale: float
    value_seed: int
    q_prescale: float = 1.0
    note: str = ""
    extra: dict = field(default_factory=dict)
    shard_cut: list | None = None   # per sequence: 0 = contiguous slice, 1 = chunks r and 2N-1-r of 2N


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bf16, returned as uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rnd = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + rnd) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def lognormal_lengths(rng, median, sigma, lo, hi, budget):
    """Draw clip(round(exp(N(ln median, sigma))), lo, hi) until the budget is
    full; the draw that would overflow is cut to the remainder (dropped if
    that is below ``lo``)."""
    out, left = [], int(budget)
    while left > 0:
        L = int(np.clip(np.rint(np.exp(rng.normal(np.log(median), sigma))), lo, hi))
        if L > left:
            if left >= lo:
                out.append(left)
            break
        out.append(L)
        left -= L
    return out


def config(n: int, shard_index: int | None = None) -> Workload:
    """The five benchmark micro-batches (n = 1..5).

    1: tiny, 4 sequences {37,128,256,511}, 4/4 heads, d=64, Q pre-scaled by 1/8.
    2: Qwen2.5-0.5B-shaped (14/2 heads, d=64), 16,384-token lognormal mix.
    3: Llama-3-8B-shaped (32/8, d=128), one 24,576 sequence + 8,192 short tokens.
    4: Llama-3-8B-shaped, query shard (index 7 of 8 by default) of a 131,072
       sequence + 8,192 short tokens.
    5: Qwen2.5-7B-shaped (28/4, d=128), bimodal 65,536-token mix + shard 3 of 4
       of a 65,536 sequence.
    """
    if n == 1:
        S = [37, 128, 256, 511]
        return Workload("config1_tiny", S, [1] * 4, [0] * 4, 4, 4, 64, 1.0, 0, q_prescale=0.125)
    rng = np.random.Generator(np.random.PCG64(n))
    if n == 2:
        S = lognormal_lengths(rng, 600, 1.0, 16, 8192, 16384)
        return Workload("config2_qwen0.5b_16k", S, [1] * len(S), [0] * len(S), 14, 2, 64,
                        64 ** -0.5, 1000 + n)
    if n == 3:
        S = [24576] + lognormal_lengths(rng, 800, 0.8, 32, 4096, 8192)
        return Workload("config3_llama8b_32k", S, [1] * len(S), [0] * len(S), 32, 8, 128,
                        128 ** -0.5, 1000 + n)
    if n == 4:
        r = 7 if shard_index is None else int(shard_index)
        short = lognormal_lengths(rng, 1000, 0.8, 64, 4096, 8192)
        S = [131072] + short
        return Workload(f"config4_llama8b_shard{r}of8", S, [8] + [1] * len(short),
                        [r] + [0] * len(short), 32, 8, 128, 128 ** -0.5, 1000 + n)
    if n == 5:
        longs = []
        while sum(longs) < 26214:
            longs.append(int(rng.integers(16384, 49153)))
        short = lognormal_lengths(rng, 1000, 0.9, 32, 8192, 65536 - sum(longs))
        r = 3 if shard_index is None else int(shard_index)
        S = [65536] + longs + short
        return Workload(f"config5_qwen7b_bimodal_shard{r}of4", S, [4] + [1] * (len(S) - 1),
                        [r] + [0] * (len(S) - 1), 28, 4, 128, 128 ** -0.5, 1000 + n)
    raise ValueError("config number must be 1..5")


def scaled_shard_twin(seq_len=16384, degree=8, index=7, heads=(8, 2), head_dim=128,
                      short_budget=1024, seed=44) -> Workload:
    """A small micro-batch with the structure of config 4 (one sharded long
    sequence plus short local ones) that the oracle can check exhaustively."""
    rng = np.random.Generator(np.random.PCG64(seed))
    short = lognormal_lengths(rng, 200, 0.8, 16, 512, short_budget)
    S = [seq_len] + short
    return Workload(f"shard_twin_{seq_len}_{index}of{degree}", S, [degree] + [1] * len(short),
                    [index] + [0] * len(short), heads[0], heads[1], head_dim,
                    head_dim ** -0.5, seed + 1000)


def make_values(w: Workload, total_q: int, total_k: int) -> dict:
    """bf16 bit patterns (uint16) of Q, K, V, dO: i.i.d. N(0,1) drawn in float32
    (Q times ``q_prescale``), rounded to nearest even."""
    rng = np.random.Generator(np.random.PCG64(w.value_seed))
    d = w.head_dim
    out = {}
    for name, shape in (("q", (total_q, w.num_q_heads, d)), ("k", (total_k, w.num_kv_heads, d)),
                        ("v", (total_k, w.num_kv_heads, d)), ("do", (total_q, w.num_q_heads, d))):
        x = rng.standard_normal(shape, dtype=np.float32)
        if name == "q" and w.q_prescale != 1.0:
            x *= np.float32(w.q_prescale)
        out[name] = f32_to_bf16_bits(x)
    return out


# The paper's Table 1: share of sequences below 1K / 4K / 8K / 32K / 128K tokens and
# the longest sequence, per corpus.  The corpora themselves are not available here;
# `table1_lengths` draws from a piecewise log-uniform density with exactly these shares.
TABLE1_EDGES = (16, 1024, 4096, 8192, 32768, 131072)
TABLE1 = {
    "wikipedia": ((0.8788, 0.9934, 0.9992, 0.9999, 1.0), 78 * 1024),
    "lmsyschat1m": ((0.8712, 0.9935, 0.9987, 0.9998, 0.9999), 1643 * 1024),
    "chatqa2_long_sft": ((0.2192, 0.3148, 0.4043, 0.9986, 1.0), 99 * 1024),
}

# (hidden h, hidden_kv h_kv, query heads, key/value heads, head_dim) of the model shapes
# the paper trains (Qwen2.5-0.5B, Qwen2.5-7B) and of Llama-3-8B.
MODEL_SHAPES = {
    "qwen2.5-0.5b": (896, 128, 14, 2, 64),
    "qwen2.5-7b": (3584, 512, 28, 4, 128),
    "llama-3-8b": (4096, 1024, 32, 8, 128),
}


def table1_lengths(rng, dataset: str, count: int | None = None, budget: int | None = None,
                   longest: int | None = None):
    """Sequence lengths with the Table 1 shares of `dataset`: a bucket is chosen with
    the table's probability, the length log-uniformly inside it (the tail beyond 128K
    reaches to the corpus' longest sequence, or to `longest`).  Draw `count` lengths,
    or as many as fit a `budget` of tokens: the first draw that would overflow ends the
    batch and is dropped (redrawn while the batch is still empty)."""
    cdf, cap = TABLE1[dataset]
    cap = min(cap, longest) if longest else cap
    edges = list(TABLE1_EDGES) + [max(cap, TABLE1_EDGES[-1] + 1)]
    out, left = [], budget
    while (count is None or len(out) < count) and (left is None or left > 0):
        u = rng.random()
        b = int(np.searchsorted(np.asarray(cdf), u, side="right"))
        lo, hi = edges[b], edges[b + 1]
        L = int(min(np.exp(rng.uniform(np.log(lo), np.log(hi))), cap))
        if left is not None:
            if L > left:
                if out:
                    break
                continue
            left -= L
        out.append(L)
    return out

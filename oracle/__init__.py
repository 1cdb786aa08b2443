"""CPU fp64 oracle for packed varlen causal attention -- TEST INFRASTRUCTURE ONLY.

Thin ctypes/numpy front end over ``skrull_oracle.c`` (plain C, double
precision, the written-out definition).  Only ``tests/``, the smoke check and
the benchmark's ``cpu_baseline`` leg may import this package.  It shares no
code with the HIP library and imports nothing from it.

Conventions (identical to what the C file documents):
  Q, dO : float32 [Tq, Hq, d]   (bf16 values widened exactly)
  K, V  : float32 [Tk, Hkv, d]
  a *descriptor* is the dict returned by :func:`ranges`.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "skrull_oracle.c")
_LIB = os.path.join(_HERE, "libskrull_oracle.so")
_lib = None

_i32p = ctypes.POINTER(ctypes.c_int32)
_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math: plain IEEE double)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_ranges.restype = ctypes.c_int
        lib.oracle_attended_pairs.restype = ctypes.c_int64
        lib.oracle_fwd_items.restype = ctypes.c_int32
        lib.oracle_dkv_items.restype = ctypes.c_int32
        lib.oracle_num_threads.restype = ctypes.c_int32
        lib.oracle_fwd_rows.restype = None
        lib.oracle_bwd_dq_rows.restype = None
        lib.oracle_bwd_dkv_cols.restype = None
        _lib = lib
    return _lib


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _p(a, ty):
    return a.ctypes.data_as(ty)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


# --------------------------------------------------------------------------
# integer part
# --------------------------------------------------------------------------
def ranges(seq_len, shard_degree=None, shard_index=None, shard_cut=None) -> dict:
    """Query segments and packed offsets (paper Eq. 8 slices).  A sequence cut the
    contiguous way (shard_cut 0, the default) is one segment; one cut the load-balanced
    way (shard_cut 1: chunks r and 2N-1-r of 2N) is two consecutive segments that share
    one key/value prefix.  Every array of the result is per SEGMENT."""
    S = _i32(seq_len)
    K = S.shape[0]
    N = _i32(np.ones(K) if shard_degree is None else shard_degree)
    r = _i32(np.zeros(K) if shard_index is None else shard_index)
    z = _i32(np.zeros(K) if shard_cut is None else shard_cut)
    out = {n: np.zeros(2 * K, np.int32) for n in ("q_begin", "q_len", "kv_len", "shares_kv")}
    out["cu_q"] = np.zeros(2 * K + 1, np.int32)
    out["cu_k"] = np.zeros(2 * K + 1, np.int32)
    ns = _load().oracle_ranges(ctypes.c_int32(K), _p(S, _i32p), _p(N, _i32p), _p(r, _i32p),
                               _p(z, _i32p),
                               _p(out["q_begin"], _i32p), _p(out["q_len"], _i32p),
                               _p(out["kv_len"], _i32p), _p(out["cu_q"], _i32p),
                               _p(out["cu_k"], _i32p), _p(out["shares_kv"], _i32p))
    if ns < 0:
        raise ValueError("oracle_ranges: invalid problem")
    for n in ("q_begin", "q_len", "kv_len", "shares_kv"):
        out[n] = np.ascontiguousarray(out[n][:ns])
    out["cu_q"] = np.ascontiguousarray(out["cu_q"][:ns + 1])
    out["cu_k"] = np.ascontiguousarray(out["cu_k"][:ns + 1])
    out["num_seqs"] = ns          # number of segments: the length of the arrays above
    out["total_q"] = int(out["cu_q"][ns])
    out["total_k"] = int(out["cu_k"][ns])
    return out


def attended_pairs(desc: dict) -> int:
    return int(_load().oracle_attended_pairs(ctypes.c_int32(desc["num_seqs"]),
                                             _p(desc["q_begin"], _i32p), _p(desc["q_len"], _i32p)))


def fwd_items(desc: dict, block_m: int, block_n: int) -> np.ndarray:
    """Forward/dQ work list, int32 [n, 4] = {seq, q_block, q_row, n_kv}."""
    lib = _load()
    K = ctypes.c_int32(desc["num_seqs"])
    args = (K, _p(desc["q_begin"], _i32p), _p(desc["q_len"], _i32p), _p(desc["cu_q"], _i32p),
            ctypes.c_int32(block_m), ctypes.c_int32(block_n))
    n = lib.oracle_fwd_items(*args, None)
    items = np.zeros((n, 4), np.int32)
    lib.oracle_fwd_items(*args, _p(items, _i32p))
    return items


def dkv_items(desc: dict, block_m: int, block_n: int) -> np.ndarray:
    """dK/dV work list, int32 [n, 4] = {seq, kv_block, m0, n_q}."""
    lib = _load()
    K = ctypes.c_int32(desc["num_seqs"])
    args = (K, _p(desc["q_begin"], _i32p), _p(desc["q_len"], _i32p), _p(desc["kv_len"], _i32p),
            _p(desc["shares_kv"], _i32p), ctypes.c_int32(block_m), ctypes.c_int32(block_n))
    n = lib.oracle_dkv_items(*args, None)
    items = np.zeros((n, 4), np.int32)
    lib.oracle_dkv_items(*args, _p(items, _i32p))
    return items


# --------------------------------------------------------------------------
# floating part
# --------------------------------------------------------------------------
def all_row_entries(desc: dict, num_heads: int, seqs=None):
    """(seq, head, row) triples for every query row of the given sequences."""
    seqs = range(desc["num_seqs"]) if seqs is None else seqs
    s, h, i = [], [], []
    for k in seqs:
        n = int(desc["q_len"][k])
        hh, ii = np.meshgrid(np.arange(num_heads, dtype=np.int32),
                             np.arange(n, dtype=np.int32), indexing="ij")
        s.append(np.full(hh.size, k, np.int32))
        h.append(hh.ravel())
        i.append(ii.ravel())
    if not s:
        z = np.zeros(0, np.int32)
        return z, z.copy(), z.copy()
    return np.concatenate(s), np.concatenate(h), np.concatenate(i)


def all_col_entries(desc: dict, num_kv_heads: int, seqs=None):
    """(seq, kv head, key position) triples for every KV row of the given sequences."""
    seqs = range(desc["num_seqs"]) if seqs is None else seqs
    s, c, j = [], [], []
    for k in seqs:
        n = int(desc["kv_len"][k])
        cc, jj = np.meshgrid(np.arange(num_kv_heads, dtype=np.int32),
                             np.arange(n, dtype=np.int32), indexing="ij")
        s.append(np.full(cc.size, k, np.int32))
        c.append(cc.ravel())
        j.append(jj.ravel())
    if not s:
        z = np.zeros(0, np.int32)
        return z, z.copy(), z.copy()
    return np.concatenate(s), np.concatenate(c), np.concatenate(j)


def _shape(q, k):
    Tq, Hq, d = q.shape
    Tk, Hkv, d2 = k.shape
    assert d == d2 and Hq % Hkv == 0
    return Tq, Hq, Tk, Hkv, d


def fwd_rows(q, k, v, desc, scale, entries):
    """O [n, d] and LSE [n] (float64) for the listed (seq, head, row) triples."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    Tq, Hq, Tk, Hkv, d = _shape(q, k)
    assert Tq == desc["total_q"] and Tk == desc["total_k"] and v.shape == k.shape
    s, h, i = (_i32(e) for e in entries)
    n = s.shape[0]
    O = np.zeros((n, d), np.float64)
    LSE = np.zeros(n, np.float64)
    _load().oracle_fwd_rows(_p(q, _f32p), _p(k, _f32p), _p(v, _f32p),
                            ctypes.c_int32(Hq), ctypes.c_int32(Hkv), ctypes.c_int32(d),
                            ctypes.c_double(scale),
                            _p(desc["q_begin"], _i32p), _p(desc["cu_q"], _i32p),
                            _p(desc["cu_k"], _i32p),
                            ctypes.c_int64(n), _p(s, _i32p), _p(h, _i32p), _p(i, _i32p),
                            _p(O, _f64p), _p(LSE, _f64p))
    return O, LSE


def bwd_dq_rows(q, k, v, do, desc, scale, entries):
    """dQ [n, d] and D [n] (float64) for the listed (seq, head, row) triples."""
    q, k, v, do = _f32(q), _f32(k), _f32(v), _f32(do)
    Tq, Hq, Tk, Hkv, d = _shape(q, k)
    assert Tq == desc["total_q"] and Tk == desc["total_k"] and do.shape == q.shape
    s, h, i = (_i32(e) for e in entries)
    n = s.shape[0]
    dQ = np.zeros((n, d), np.float64)
    D = np.zeros(n, np.float64)
    _load().oracle_bwd_dq_rows(_p(q, _f32p), _p(k, _f32p), _p(v, _f32p), _p(do, _f32p),
                               ctypes.c_int32(Hq), ctypes.c_int32(Hkv), ctypes.c_int32(d),
                               ctypes.c_double(scale),
                               _p(desc["q_begin"], _i32p), _p(desc["cu_q"], _i32p),
                               _p(desc["cu_k"], _i32p),
                               ctypes.c_int64(n), _p(s, _i32p), _p(h, _i32p), _p(i, _i32p),
                               _p(dQ, _f64p), _p(D, _f64p))
    return dQ, D


def delta_rows(do_rows, o_rows):
    """D [n] (float64) from rows of dO and of the forward's O: D_i = sum_t dO_i[t] * O_i[t],
    the row term of the softmax gradient dS_ij = P_ij (dP_ij - D_i).  ``o_rows`` is the
    float64 O that :func:`fwd_rows` returned for the same (seq, head, row) triples and
    ``do_rows`` the matching rows of dO; bwd_dq_rows returns the same D (pinned against it
    in tests/test_oracle_attention.py) but recomputes the whole row to get it."""
    do_rows = np.asarray(do_rows, np.float64)
    o_rows = np.asarray(o_rows, np.float64)
    assert do_rows.shape == o_rows.shape and do_rows.ndim == 2
    D = np.zeros(do_rows.shape[0], np.float64)
    for t in range(do_rows.shape[1]):
        D += do_rows[:, t] * o_rows[:, t]
    return D


def bwd_dkv_cols(q, k, v, do, lse_full, d_full, desc, scale, entries):
    """dK, dV [n, d] (float64) for the listed (seq, kv head, key position) triples.

    ``lse_full`` / ``d_full`` are float64 [Hq, Tq]; only cells the listed
    columns can see need to be valid."""
    q, k, v, do = _f32(q), _f32(k), _f32(v), _f32(do)
    Tq, Hq, Tk, Hkv, d = _shape(q, k)
    lse_full = np.ascontiguousarray(lse_full, np.float64)
    d_full = np.ascontiguousarray(d_full, np.float64)
    assert lse_full.shape == (Hq, Tq) and d_full.shape == (Hq, Tq)
    s, c, j = (_i32(e) for e in entries)
    n = s.shape[0]
    dK = np.zeros((n, d), np.float64)
    dV = np.zeros((n, d), np.float64)
    _load().oracle_bwd_dkv_cols(_p(q, _f32p), _p(k, _f32p), _p(v, _f32p), _p(do, _f32p),
                                _p(lse_full, _f64p), _p(d_full, _f64p), ctypes.c_int64(Tq),
                                ctypes.c_int32(Hq), ctypes.c_int32(Hkv), ctypes.c_int32(d),
                                ctypes.c_double(scale),
                                _p(desc["q_begin"], _i32p), _p(desc["q_len"], _i32p),
                                _p(desc["cu_q"], _i32p), _p(desc["cu_k"], _i32p),
                                ctypes.c_int64(n), _p(s, _i32p), _p(c, _i32p), _p(j, _i32p),
                                _p(dK, _f64p), _p(dV, _f64p))
    return dK, dV


def attention_fwd(q, k, v, desc, scale):
    """Whole micro-batch forward: O [Tq, Hq, d], LSE [Hq, Tq] (float64)."""
    Tq, Hq, Tk, Hkv, d = _shape(np.asarray(q), np.asarray(k))
    ent = all_row_entries(desc, Hq)
    o, lse = fwd_rows(q, k, v, desc, scale, ent)
    rows = desc["cu_q"][ent[0]] + ent[2]
    O = np.zeros((Tq, Hq, d), np.float64)
    LSE = np.zeros((Hq, Tq), np.float64)
    O[rows, ent[1]] = o
    LSE[ent[1], rows] = lse
    return O, LSE


def attention_bwd(q, k, v, do, desc, scale):
    """Whole micro-batch backward: dQ [Tq,Hq,d], dK, dV [Tk,Hkv,d], D [Hq,Tq] (float64)."""
    Tq, Hq, Tk, Hkv, d = _shape(np.asarray(q), np.asarray(k))
    ent = all_row_entries(desc, Hq)
    rows = desc["cu_q"][ent[0]] + ent[2]
    _, lse = fwd_rows(q, k, v, desc, scale, ent)
    dq, dd = bwd_dq_rows(q, k, v, do, desc, scale, ent)
    dQ = np.zeros((Tq, Hq, d), np.float64)
    LSE = np.zeros((Hq, Tq), np.float64)
    D = np.zeros((Hq, Tq), np.float64)
    dQ[rows, ent[1]] = dq
    LSE[ent[1], rows] = lse
    D[ent[1], rows] = dd
    cent = all_col_entries(desc, Hkv)
    dk, dv = bwd_dkv_cols(q, k, v, do, LSE, D, desc, scale, cent)
    crow = desc["cu_k"][cent[0]] + cent[2]
    dK = np.zeros((Tk, Hkv, d), np.float64)
    dV = np.zeros((Tk, Hkv, d), np.float64)
    # += : two segments that share a key/value prefix both contribute to its rows
    np.add.at(dK, (crow, cent[1]), dk)
    np.add.at(dV, (crow, cent[1]), dv)
    return dQ, dK, dV, D

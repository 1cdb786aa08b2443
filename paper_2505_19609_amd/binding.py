"""ctypes binding of libskrull_attn.so: same names as the C ABI, argument
marshalling only.  Tensors are torch CUDA(HIP) tensors used purely as device
memory; every step of the path runs in the library's kernels.  There is no CPU
fallback: a missing library raises."""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libskrull_attn.so")

SKRULL_OK, SKRULL_EINVAL, SKRULL_ENOMEM, SKRULL_EHIP, SKRULL_EUNSUPPORTED, SKRULL_ESCHED = 0, -1, -2, -3, -4, -5
(ARRAY_CU_Q, ARRAY_CU_K, ARRAY_Q_BEGIN, ARRAY_Q_LEN, ARRAY_KV_LEN, ARRAY_FWD_ITEMS, ARRAY_DKV_ITEMS,
 ARRAY_SHARES_KV) = range(8)
CUT_CONTIGUOUS, CUT_TWO_CHUNKS = 0, 1

EXPORTED_SYMBOLS = ("skrull_attn_plan", "skrull_attn_plan_info", "skrull_attn_plan_export",
                    "skrull_attn_fwd", "skrull_attn_bwd", "skrull_attn_bwd_static", "skrull_attn_plan_destroy",
                    "skrull_attn_strerror", "skrull_attn_profile", "skrull_attn_profile_read",
                    "skrull_attn_mfma_ceiling", "skrull_attn_trace", "skrull_attn_trace_layout",
                    "skrull_dacp_schedule", "skrull_dacp_rank_batch",
                    "skrull_gds_binpack", "skrull_gds_schedule", "skrull_gds_micro_batch")


class Problem(ctypes.Structure):
    _fields_ = [("num_seqs", ctypes.c_int32),
                ("seq_len", ctypes.POINTER(ctypes.c_int32)),
                ("shard_degree", ctypes.POINTER(ctypes.c_int32)),
                ("shard_index", ctypes.POINTER(ctypes.c_int32)),
                ("num_q_heads", ctypes.c_int32),
                ("num_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32),
                ("softmax_scale", ctypes.c_float),
                ("block_m", ctypes.c_int32),
                ("block_n", ctypes.c_int32),
                ("shard_cut", ctypes.POINTER(ctypes.c_int32)),
                ("head_split", ctypes.c_int32), ("wg_query_rows", ctypes.c_int32)]


class PlanInfo(ctypes.Structure):
    _fields_ = [("num_seqs", ctypes.c_int32), ("num_q_heads", ctypes.c_int32),
                ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("block_m", ctypes.c_int32), ("block_n", ctypes.c_int32),
                ("total_q", ctypes.c_int32), ("total_k", ctypes.c_int32),
                ("n_fwd_items", ctypes.c_int32), ("n_dkv_items", ctypes.c_int32),
                ("attended_pairs", ctypes.c_int64), ("useful_flops_fwd", ctypes.c_int64),
                ("useful_flops_bwd", ctypes.c_int64), ("bwd_workspace_bytes", ctypes.c_int64),
                ("num_segments", ctypes.c_int32), ("head_split", ctypes.c_int32),
                ("wg_query_rows", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class FlopsModel(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_int64), ("hidden_kv", ctypes.c_int64), ("batch", ctypes.c_int64)]


class SkrullError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"skrull_attn error {code}: {msg}")
        self.code = code


_lib = None


def lib():
    """Load the in-tree HIP library; raise loudly if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run __graft_entry__.build() "
                               "(python -m paper_2505_19609_amd.build); there is no fallback path")
        # PyTorch ships its own HIP runtime; loading it first lets this library's
        # libamdhip64 dependency resolve to that same copy, so device pointers and
        # streams made by torch are valid in our calls (two runtimes in one process
        # do not see each other's devices).
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp = ctypes.c_void_p
        L.skrull_attn_plan.argtypes = [ctypes.POINTER(Problem), vp, ctypes.POINTER(vp)]
        L.skrull_attn_plan.restype = ctypes.c_int
        L.skrull_attn_plan_info.argtypes = [vp, ctypes.POINTER(PlanInfo)]
        L.skrull_attn_plan_info.restype = ctypes.c_int
        L.skrull_attn_plan_export.argtypes = [vp, ctypes.c_int, vp, ctypes.c_size_t]
        L.skrull_attn_plan_export.restype = ctypes.c_int
        L.skrull_attn_fwd.argtypes = [vp] * 7
        L.skrull_attn_fwd.restype = ctypes.c_int
        L.skrull_attn_bwd.argtypes = [vp] * 11 + [ctypes.c_size_t, vp]
        L.skrull_attn_bwd.restype = ctypes.c_int
        L.skrull_attn_bwd_static.argtypes = [vp] * 11
        L.skrull_attn_bwd_static.restype = ctypes.c_int
        L.skrull_attn_plan_destroy.argtypes = [vp]
        L.skrull_attn_plan_destroy.restype = None
        L.skrull_attn_strerror.argtypes = [ctypes.c_int]
        L.skrull_attn_strerror.restype = ctypes.c_char_p
        L.skrull_attn_profile.argtypes = [ctypes.c_int]
        L.skrull_attn_profile.restype = ctypes.c_int
        L.skrull_attn_profile_read.argtypes = [ctypes.POINTER(ctypes.c_float)]
        L.skrull_attn_profile_read.restype = ctypes.c_int
        L.skrull_attn_mfma_ceiling.argtypes = [vp, ctypes.POINTER(ctypes.c_float)]
        L.skrull_attn_mfma_ceiling.restype = ctypes.c_int
        i32p = ctypes.POINTER(ctypes.c_int32)
        L.skrull_attn_trace.argtypes = [vp, ctypes.c_size_t]
        L.skrull_attn_trace.restype = ctypes.c_int
        L.skrull_attn_trace_layout.argtypes = [vp, i32p, i32p]
        L.skrull_attn_trace_layout.restype = ctypes.c_int
        L.skrull_dacp_schedule.argtypes = [ctypes.c_int32, i32p, ctypes.c_int64, ctypes.c_int32,
                                           ctypes.POINTER(FlopsModel), i32p]
        L.skrull_dacp_schedule.restype = ctypes.c_int
        L.skrull_dacp_rank_batch.argtypes = [ctypes.c_int32, i32p, i32p, ctypes.c_int32, ctypes.c_int32,
                                             i32p, i32p, i32p, i32p, i32p]
        L.skrull_dacp_rank_batch.restype = ctypes.c_int
        L.skrull_gds_binpack.argtypes = [ctypes.c_int32, i32p, ctypes.c_int32, ctypes.POINTER(FlopsModel), i32p]
        L.skrull_gds_binpack.restype = ctypes.c_int
        L.skrull_gds_schedule.argtypes = [ctypes.c_int32, i32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                          ctypes.c_int32, ctypes.POINTER(FlopsModel), i32p, i32p, i32p, i32p]
        L.skrull_gds_schedule.restype = ctypes.c_int
        L.skrull_gds_micro_batch.argtypes = [ctypes.c_int32, i32p, i32p, ctypes.c_int32, i32p, i32p]
        L.skrull_gds_micro_batch.restype = ctypes.c_int
        _lib = L
    return _lib


def skrull_attn_strerror(code: int) -> str:
    return lib().skrull_attn_strerror(code).decode()


def _check(rc: int):
    if rc != SKRULL_OK:
        raise SkrullError(rc, skrull_attn_strerror(rc))


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(int(getattr(stream, "cuda_stream", stream)))


class Plan:
    """Owner of a ``skrull_attn_plan_t*``."""

    def __init__(self, handle, info: PlanInfo):
        self.handle = handle
        self.info = info

    def __getattr__(self, name):
        return getattr(self.info, name)

    def destroy(self):
        if self.handle:
            lib().skrull_attn_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def skrull_attn_plan(seq_len, shard_degree, shard_index, num_q_heads, num_kv_heads, head_dim,
                     softmax_scale, block_m=0, block_n=0, stream=None, raw_stream=None,
                     shard_cut=None, head_split=0, wg_query_rows=0) -> Plan:
    S = np.ascontiguousarray(seq_len, dtype=np.int32)
    N = np.ascontiguousarray(shard_degree, dtype=np.int32)
    R = np.ascontiguousarray(shard_index, dtype=np.int32)
    Z = None if shard_cut is None else np.ascontiguousarray(shard_cut, dtype=np.int32)
    if not (S.shape == N.shape == R.shape and S.ndim == 1 and (Z is None or Z.shape == S.shape)):
        raise SkrullError(SKRULL_EINVAL, "seq_len / shard_degree / shard_index / shard_cut must be 1-D and equally long")
    i32p = ctypes.POINTER(ctypes.c_int32)
    prob = Problem(int(S.shape[0]), S.ctypes.data_as(i32p), N.ctypes.data_as(i32p),
                   R.ctypes.data_as(i32p), num_q_heads, num_kv_heads, head_dim,
                   float(softmax_scale), block_m, block_n,
                   None if Z is None else Z.ctypes.data_as(i32p), int(head_split), int(wg_query_rows))
    handle = ctypes.c_void_p()
    st = ctypes.c_void_p(raw_stream) if raw_stream is not None else _stream_ptr(stream)
    _check(lib().skrull_attn_plan(ctypes.byref(prob), st, ctypes.byref(handle)))
    info = PlanInfo()
    _check(lib().skrull_attn_plan_info(handle, ctypes.byref(info)))
    return Plan(handle, info)


def skrull_attn_plan_info(plan: Plan) -> PlanInfo:
    info = PlanInfo()
    _check(lib().skrull_attn_plan_info(plan.handle, ctypes.byref(info)))
    return info


def skrull_attn_plan_export(plan: Plan, which: int) -> np.ndarray:
    K = plan.info.num_segments
    shape = {ARRAY_CU_Q: (K + 1,), ARRAY_CU_K: (K + 1,), ARRAY_Q_BEGIN: (K,), ARRAY_Q_LEN: (K,),
             ARRAY_KV_LEN: (K,), ARRAY_SHARES_KV: (K,), ARRAY_FWD_ITEMS: (plan.info.n_fwd_items, 4),
             ARRAY_DKV_ITEMS: (plan.info.n_dkv_items, 4)}[which]
    out = np.zeros(shape, np.int32)
    _check(lib().skrull_attn_plan_export(plan.handle, which, out.ctypes.data_as(ctypes.c_void_p),
                                         out.nbytes))
    return out


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def skrull_attn_fwd(plan: Plan, q, k, v, o, lse, stream=None):
    _check(lib().skrull_attn_fwd(plan.handle, _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse),
                                 _stream_ptr(stream)))


def skrull_attn_bwd(plan: Plan, q, k, v, o, lse, d_o, dq, dk, dv, workspace, stream=None):
    _check(lib().skrull_attn_bwd(plan.handle, _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse),
                                 _ptr(d_o), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream_ptr(stream)))


STATIC_SCRATCH_BYTES = 32 * 1024 * 1024


def skrull_attn_bwd_static(plan: Plan, q, k, v, o, lse, d_o, dq, dk, dv, stream=None):
    """skrull_attn_bwd on the library's static workspace (no allocation anywhere)."""
    _check(lib().skrull_attn_bwd_static(plan.handle, _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse),
                                        _ptr(d_o), _ptr(dq), _ptr(dk), _ptr(dv), _stream_ptr(stream)))


def skrull_attn_profile(enable: bool):
    _check(lib().skrull_attn_profile(int(bool(enable))))


def skrull_attn_profile_read():
    """Kernel durations (ms) of the last forward / backward: [fwd, 0, dkv, dq] (the second
    slot was a separate rowsum(dO*O) kernel; the dQ kernel forms it now)."""
    ms = (ctypes.c_float * 4)()
    _check(lib().skrull_attn_profile_read(ms))
    return [float(x) for x in ms]


def skrull_attn_trace(records=None):
    """Switch the per-workgroup trace on (records: a zeroed torch uint8 CUDA tensor) or off (None)."""
    if records is None:
        _check(lib().skrull_attn_trace(None, 0))
    else:
        _check(lib().skrull_attn_trace(_ptr(records), records.numel() * records.element_size()))


def skrull_attn_trace_layout(plan: Plan):
    """(first_record[3], num_records[3]) of the forward, dQ and dK/dV kernels of `plan`."""
    first, num = (ctypes.c_int32 * 3)(), (ctypes.c_int32 * 3)()
    _check(lib().skrull_attn_trace_layout(plan.handle, first, num))
    return [int(x) for x in first], [int(x) for x in num]


def skrull_attn_mfma_ceiling(stream=None) -> float:
    """TFLOP/s this GPU sustains on bf16 MFMAs alone (measurement aid)."""
    out = ctypes.c_float(0.0)
    _check(lib().skrull_attn_mfma_ceiling(_stream_ptr(stream), ctypes.byref(out)))
    return float(out.value)


def skrull_dacp_schedule(seq_len, bucket_size, cp_degree, hidden, hidden_kv, batch=1) -> np.ndarray:
    """ret[K]: the rank that keeps sequence k whole, or -1 if it is distributed.
    Raises SkrullError(SKRULL_ESCHED) when the micro-batch does not fit."""
    S = np.ascontiguousarray(seq_len, dtype=np.int32)
    if S.ndim != 1:
        raise SkrullError(SKRULL_EINVAL, "seq_len must be 1-D")
    ret = np.zeros(S.shape[0], np.int32)
    i32p = ctypes.POINTER(ctypes.c_int32)
    model = FlopsModel(int(hidden), int(hidden_kv), int(batch))
    _check(lib().skrull_dacp_schedule(int(S.shape[0]), S.ctypes.data_as(i32p), int(bucket_size),
                                      int(cp_degree), ctypes.byref(model), ret.ctypes.data_as(i32p)))
    return ret


def skrull_dacp_rank_batch(seq_len, ret, cp_degree, rank):
    """(seq_len, shard_degree, shard_index, source) of rank `rank`'s micro-batch."""
    S = np.ascontiguousarray(seq_len, dtype=np.int32)
    R = np.ascontiguousarray(ret, dtype=np.int32)
    if S.ndim != 1 or S.shape != R.shape:
        raise SkrullError(SKRULL_EINVAL, "seq_len / ret must be 1-D and equally long")
    K = int(S.shape[0])
    out = [np.zeros(max(K, 1), np.int32) for _ in range(4)]
    n = ctypes.c_int32(0)
    i32p = ctypes.POINTER(ctypes.c_int32)
    _check(lib().skrull_dacp_rank_batch(K, S.ctypes.data_as(i32p), R.ctypes.data_as(i32p),
                                        int(cp_degree), int(rank), *[o.ctypes.data_as(i32p) for o in out],
                                        ctypes.byref(n)))
    return tuple(o[:n.value].copy() for o in out)


def _lengths(seq_len) -> np.ndarray:
    S = np.ascontiguousarray(seq_len, dtype=np.int32)
    if S.ndim != 1:
        raise SkrullError(SKRULL_EINVAL, "seq_len must be 1-D")
    return S


def skrull_gds_binpack(seq_len, dp_world_size, hidden, hidden_kv, batch=1) -> np.ndarray:
    """dp_bin[K]: the DP rank of every sequence of the global batch."""
    S = _lengths(seq_len)
    out = np.zeros(S.shape[0], np.int32)
    i32p = ctypes.POINTER(ctypes.c_int32)
    model = FlopsModel(int(hidden), int(hidden_kv), int(batch))
    _check(lib().skrull_gds_binpack(int(S.shape[0]), S.ctypes.data_as(i32p), int(dp_world_size),
                                    ctypes.byref(model), out.ctypes.data_as(i32p)))
    return out


def skrull_gds_schedule(seq_len, bucket_size, cp_degree, dp_world_size, dp_rank, hidden, hidden_kv, batch=1):
    """(dp_bin[K], micro_batch[K], ret[K], num_micro_batches) for DP rank `dp_rank`."""
    S = _lengths(seq_len)
    K = int(S.shape[0])
    bins, mb, ret = (np.zeros(K, np.int32) for _ in range(3))
    n = ctypes.c_int32(0)
    i32p = ctypes.POINTER(ctypes.c_int32)
    model = FlopsModel(int(hidden), int(hidden_kv), int(batch))
    _check(lib().skrull_gds_schedule(K, S.ctypes.data_as(i32p), int(bucket_size), int(cp_degree),
                                     int(dp_world_size), int(dp_rank), ctypes.byref(model),
                                     bins.ctypes.data_as(i32p), mb.ctypes.data_as(i32p),
                                     ret.ctypes.data_as(i32p), ctypes.byref(n)))
    return bins, mb, ret, int(n.value)


def skrull_gds_micro_batch(seq_len, micro_batch, index) -> np.ndarray:
    """Positions (caller's list) of the members of micro-batch `index`, ascending length."""
    S = _lengths(seq_len)
    M = np.ascontiguousarray(micro_batch, dtype=np.int32)
    if M.shape != S.shape:
        raise SkrullError(SKRULL_EINVAL, "seq_len / micro_batch must be equally long")
    out = np.zeros(max(int(S.shape[0]), 1), np.int32)
    n = ctypes.c_int32(0)
    i32p = ctypes.POINTER(ctypes.c_int32)
    _check(lib().skrull_gds_micro_batch(int(S.shape[0]), S.ctypes.data_as(i32p), M.ctypes.data_as(i32p),
                                        int(index), out.ctypes.data_as(i32p), ctypes.byref(n)))
    return out[:n.value].copy()

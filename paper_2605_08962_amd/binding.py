"""Python binding of libvarlen_attn.so: argument marshalling only.

Every step of the attention path runs in the library's HIP kernels.  PyTorch is used for device
memory (outputs, workspace) and for the current stream handle, nothing else.  There is no CPU or
eager fallback: if the library is missing or a call fails, this raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvarlen_attn.so")
_lib = None

VA_OK = 0
VA_ERR_BAD_CU_SEQLENS = 8


class VarlenAttnError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"varlen_attn status {status}: {message}")
        self.status = status


class Params(ctypes.Structure):
    _fields_ = [("total_tokens", ctypes.c_int32), ("num_seqs", ctypes.c_int32),
                ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("causal", ctypes.c_int32),
                ("softmax_scale", ctypes.c_float), ("max_seqlen", ctypes.c_int32), ("kv_splits", ctypes.c_int32)]


def load():
    """Load the C-ABI library (building it first only when no built library is present)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    pp = ctypes.POINTER(Params)
    lib.varlen_attn_fwd_workspace_bytes.argtypes = [pp]
    lib.varlen_attn_fwd_workspace_bytes.restype = sz
    lib.varlen_attn_bwd_workspace_bytes.argtypes = [pp]
    lib.varlen_attn_bwd_workspace_bytes.restype = sz
    lib.varlen_attn_max_work_items.argtypes = [pp, ctypes.c_int]
    lib.varlen_attn_max_work_items.restype = ctypes.c_int64
    lib.varlen_attn_fwd.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.varlen_attn_fwd.restype = ctypes.c_int
    lib.varlen_attn_fwd_static_scratch.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp]
    lib.varlen_attn_fwd_static_scratch.restype = ctypes.c_int
    lib.varlen_attn_bwd.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.varlen_attn_bwd.restype = ctypes.c_int
    lib.varlen_attn_merge.argtypes = [pp, ctypes.c_int32, vp, vp, vp, vp, vp]
    lib.varlen_attn_merge.restype = ctypes.c_int
    lib.varlen_attn_check_cu_seqlens.argtypes = [pp, vp, vp, sz, vp]
    lib.varlen_attn_check_cu_seqlens.restype = ctypes.c_int
    lib.varlen_attn_status_string.argtypes = [ctypes.c_int]
    lib.varlen_attn_status_string.restype = ctypes.c_char_p
    lib.varlen_attn_last_hip_error.argtypes = []
    lib.varlen_attn_last_hip_error.restype = ctypes.c_int
    lib.varlen_attn_balance_partition.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                                  ctypes.c_double, ctypes.c_double, vp, vp]
    lib.varlen_attn_balance_partition.restype = ctypes.c_int
    lib.varlen_attn_profile_enable.argtypes = [ctypes.c_int]
    lib.varlen_attn_profile_enable.restype = ctypes.c_int
    lib.varlen_attn_profile_read.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_double),
                                             ctypes.POINTER(ctypes.c_int64)]
    lib.varlen_attn_profile_read.restype = ctypes.c_int
    lib.varlen_attn_profile_clock_probe.argtypes = [vp]
    lib.varlen_attn_profile_clock_probe.restype = ctypes.c_int
    _lib = lib
    return lib


def status_string(status):
    return load().varlen_attn_status_string(int(status)).decode()


def _check(status):
    if status != VA_OK:
        msg = status_string(status)
        if status == 6:
            msg += f" (hipError_t {load().varlen_attn_last_hip_error()})"
        raise VarlenAttnError(status, msg)


def make_params(total_tokens, num_seqs, num_q_heads, num_kv_heads, head_dim, causal, softmax_scale, kv_splits=0,
                max_seqlen=0):
    return Params(int(total_tokens), int(num_seqs), int(num_q_heads), int(num_kv_heads), int(head_dim),
                  int(bool(causal)), float(softmax_scale), int(max_seqlen), int(kv_splits))


def _params_of(q, k, cu_seqlens, causal, softmax_scale, kv_splits=0, max_seqlen=0):
    T, Hq, D = q.shape
    return make_params(T, cu_seqlens.numel() - 1, Hq, k.shape[1], D, causal, softmax_scale, kv_splits, max_seqlen)


def _require(t, dtype, name):
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise ValueError(f"{name} must be a contiguous {dtype} tensor on the GPU")


def fwd_workspace_bytes(params):
    return int(load().varlen_attn_fwd_workspace_bytes(ctypes.byref(params)))


def bwd_workspace_bytes(params):
    return int(load().varlen_attn_bwd_workspace_bytes(ctypes.byref(params)))


def max_work_items(params, which=0):
    return int(load().varlen_attn_max_work_items(ctypes.byref(params), which))


def _stream_handle(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def varlen_attn_fwd(q, k, v, cu_seqlens, causal, softmax_scale, out=None, lse=None, workspace=None,
                    stream=None, kv_splits=0, max_seqlen=0):
    """O bf16 [T,Hq,D] and LSE fp32 [Hq,T] of packed attention; asynchronous on the stream.
    kv_splits: 0 automatic, 1 never, 2..8 workgroups sharing the keys of each query tile.
    max_seqlen: 0 unknown, else the caller's promise that no sample is longer (a hint)."""
    lib = load()
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _require(t, torch.bfloat16, n)
    _require(cu_seqlens, torch.int32, "cu_seqlens")
    p = _params_of(q, k, cu_seqlens, causal, softmax_scale, kv_splits, max_seqlen)
    if k.shape != v.shape or k.shape[0] != q.shape[0] or k.shape[2] != q.shape[2]:
        raise ValueError("k and v must be [T, Hkv, D] matching q's T and D")
    if out is None:
        out = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((q.shape[1], q.shape[0]), dtype=torch.float32, device=q.device)
    need = fwd_workspace_bytes(p)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    _check(lib.varlen_attn_fwd(ctypes.byref(p), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                               cu_seqlens.data_ptr(), out.data_ptr(), lse.data_ptr(),
                               workspace.data_ptr(), workspace.numel(), _stream_handle(stream)))
    return out, lse


STATIC_SCRATCH_BYTES = 32 << 20
VA_ERR_SCRATCH_LIMIT = 9


def varlen_attn_fwd_static_scratch(q, k, v, cu_seqlens, causal, softmax_scale, out, lse, stream=None, kv_splits=0,
                                   max_seqlen=0):
    """varlen_attn_fwd without a workspace: the scratch lives in a static device array of the library.  The
    caller passes the outputs; nothing is allocated here or in the library."""
    lib = load()
    for t, n in ((q, "q"), (k, "k"), (v, "v"), (out, "out")):
        _require(t, torch.bfloat16, n)
    _require(lse, torch.float32, "lse")
    _require(cu_seqlens, torch.int32, "cu_seqlens")
    if k.shape != v.shape or k.shape[0] != q.shape[0] or k.shape[2] != q.shape[2] or out.shape != q.shape:
        raise ValueError("k and v must be [T, Hkv, D] matching q's T and D; out must match q")
    if tuple(lse.shape) != (q.shape[1], q.shape[0]):
        raise ValueError("lse must be [Hq, T]")
    p = _params_of(q, k, cu_seqlens, causal, softmax_scale, kv_splits, max_seqlen)
    _check(lib.varlen_attn_fwd_static_scratch(ctypes.byref(p), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                              cu_seqlens.data_ptr(), out.data_ptr(), lse.data_ptr(),
                                              _stream_handle(stream)))
    return out, lse


def varlen_attn_bwd(dout, q, k, v, out, lse, cu_seqlens, causal, softmax_scale, dq=None, dk=None,
                    dv=None, workspace=None, stream=None, max_seqlen=0):
    """dQ, dK, dV (bf16) from dO and the forward's saved O and LSE; asynchronous on the stream."""
    lib = load()
    for t, n in ((dout, "dout"), (q, "q"), (k, "k"), (v, "v"), (out, "out")):
        _require(t, torch.bfloat16, n)
    _require(lse, torch.float32, "lse")
    _require(cu_seqlens, torch.int32, "cu_seqlens")
    p = _params_of(q, k, cu_seqlens, causal, softmax_scale, 0, max_seqlen)
    if dout.shape != q.shape or out.shape != q.shape or k.shape != v.shape:
        raise ValueError("dout and out must match q; k must match v")
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(v) if dv is None else dv
    need = bwd_workspace_bytes(p)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    _check(lib.varlen_attn_bwd(ctypes.byref(p), dout.data_ptr(), q.data_ptr(), k.data_ptr(),
                               v.data_ptr(), out.data_ptr(), lse.data_ptr(), cu_seqlens.data_ptr(),
                               dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), workspace.data_ptr(),
                               workspace.numel(), _stream_handle(stream)))
    return dq, dk, dv


KERNELS = {"sched": 0, "fwd": 1, "dkdv": 2, "dq": 3, "merge": 4}


def profile_enable(on=True):
    _check(load().varlen_attn_profile_enable(int(bool(on))))


def profile_read():
    """{kernel name: (total milliseconds, launches)} of the launches recorded since profile_enable."""
    out = {}
    for name, kid in KERNELS.items():
        ms, n = ctypes.c_double(0.0), ctypes.c_int64(0)
        _check(load().varlen_attn_profile_read(kid, ctypes.byref(ms), ctypes.byref(n)))
        out[name] = (ms.value, n.value)
    return out


def profile_clock_probe(counters):
    """Attach a zeroed int64 device tensor of 6 counters as the shader-clock probe, or None to detach."""
    if counters is not None and (counters.dtype != torch.int64 or counters.numel() < 6 or not counters.is_cuda
                                 or not counters.is_contiguous()):
        raise ValueError("counters must be a contiguous int64 device tensor of at least 6 elements")
    _check(load().varlen_attn_profile_clock_probe(None if counters is None else counters.data_ptr()))


def varlen_attn_merge(o_parts, lse_parts, out=None, lse=None, stream=None):
    """Merge partial results over key shards: o_parts bf16 [P,T,Hq,D], lse_parts fp32 [P,Hq,T]."""
    _require(o_parts, torch.bfloat16, "o_parts")
    _require(lse_parts, torch.float32, "lse_parts")
    P, T, Hq, D = o_parts.shape
    if tuple(lse_parts.shape) != (P, Hq, T):
        raise ValueError("lse_parts must be [P, Hq, T]")
    p = make_params(T, 1, Hq, Hq, D, False, 1.0)
    if out is None:
        out = torch.empty((T, Hq, D), dtype=torch.bfloat16, device=o_parts.device)
    if lse is None:
        lse = torch.empty((Hq, T), dtype=torch.float32, device=o_parts.device)
    _check(load().varlen_attn_merge(ctypes.byref(p), P, o_parts.data_ptr(), lse_parts.data_ptr(), out.data_ptr(),
                                    lse.data_ptr(), _stream_handle(stream)))
    return out, lse


def check_cu_seqlens(cu_seqlens, total_tokens, stream=None):
    """True if the device array obeys cu[0] = 0, non-decreasing, cu[-1] = total_tokens.  Synchronises the stream."""
    _require(cu_seqlens, torch.int32, "cu_seqlens")
    p = make_params(total_tokens, cu_seqlens.numel() - 1, 1, 1, 64, False, 1.0)
    ws = torch.empty(16, dtype=torch.uint8, device=cu_seqlens.device)
    rc = load().varlen_attn_check_cu_seqlens(ctypes.byref(p), cu_seqlens.data_ptr(), ws.data_ptr(), ws.numel(),
                                             _stream_handle(stream))
    if rc == VA_ERR_BAD_CU_SEQLENS:
        return False
    _check(rc)
    return True


PARTITION_KARMARKAR_KARP = 0
PARTITION_LPT = 1


def balance_partition(lengths, bins, method=PARTITION_KARMARKAR_KARP, equal_counts=False, lin_cost=0.0,
                      quad_cost=1.0):
    """Host-side: bin of every sample and the summed cost per bin (numpy arrays)."""
    import numpy as np
    lengths = np.ascontiguousarray(lengths, dtype=np.int32)
    bin_of = np.zeros(lengths.size, dtype=np.int32)
    bin_cost = np.zeros(max(int(bins), 0), dtype=np.float64)
    _check(load().varlen_attn_balance_partition(
        lengths.ctypes.data_as(ctypes.c_void_p), lengths.size, int(bins), int(method), int(bool(equal_counts)),
        float(lin_cost), float(quad_cost), bin_of.ctypes.data_as(ctypes.c_void_p),
        bin_cost.ctypes.data_as(ctypes.c_void_p)))
    return bin_of, bin_cost

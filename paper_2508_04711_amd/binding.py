"""ctypes binding of libhstu_attn.so: same names as the C entry points, marshalling only.

PyTorch appears here for device memory and streams alone: tensors are allocated by the
caller (or here, for outputs and workspace) and handed to the library as raw pointers.
There is no fallback path: if the HIP library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import functools
import os
from typing import Optional, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# HSTU_ATTN_LIB selects another build of the same library (A/B comparisons of kernels).
_LIB_PATH = os.environ.get("HSTU_ATTN_LIB") or os.path.join(_HERE, "libhstu_attn.so")
_lib = None

HSTU_BF16, HSTU_F32 = 0, 1
HSTU_WS_FWD, HSTU_WS_BWD, HSTU_WS_CP = 0, 1, 2
# hstu_flags (include/hstu_attn.h)
HSTU_FLAG_NO_SPLIT, HSTU_FLAG_NO_PACK, HSTU_FLAG_PACK_SHORT = 1, 2, 4
HSTU_FLAG_FWD_TILE_128, HSTU_FLAG_FWD_TILE_256, HSTU_FLAG_DKDV_ONE_WAVE = 8, 16, 32
HSTU_FLAG_BIAS_PER_PAIR = 64

# The flags every call of this module passes in hstu_attn_params.flags (0: the library's own
# choices).  Tests and benchmarks set it, preferably through the `flags` context manager.
default_flags = 0


class flags:
    """with flags(HSTU_FLAG_NO_PACK | ...): calls inside pass these hstu_flags."""

    def __init__(self, value: int):
        self.value = int(value)

    def __enter__(self):
        global default_flags
        self.saved = default_flags
        default_flags = self.value
        return self

    def __exit__(self, *exc):
        global default_flags
        default_flags = self.saved
        return False


class HstuError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, hstu_attn_status_string(status), status))


class _Params(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("num_heads", ctypes.c_int32), ("d_qk", ctypes.c_int32),
        ("d_v", ctypes.c_int32), ("max_len", ctypes.c_int32), ("alpha", ctypes.c_float),
        ("causal", ctypes.c_int32), ("dtype", ctypes.c_int32), ("total_rows", ctypes.c_int64),
        ("out_dtype", ctypes.c_int32), ("flags", ctypes.c_int32),
    ]


class _CpDesc(ctypes.Structure):
    _fields_ = [
        ("cp_size", ctypes.c_int32), ("q_rank", ctypes.c_int32), ("kv_rank", ctypes.c_int32),
        ("accumulate", ctypes.c_int32), ("q_rows", ctypes.c_int64), ("kv_rows", ctypes.c_int64),
    ]


class _TsBias(ctypes.Structure):
    _fields_ = [
        ("timestamps", ctypes.c_void_p), ("ts_weights", ctypes.c_void_p),
        ("d_ts_weights", ctypes.c_void_p), ("num_buckets", ctypes.c_int32),
        ("groups_log2", ctypes.c_int32),
    ]


class _CpTsBias(ctypes.Structure):
    _fields_ = [
        ("q_timestamps", ctypes.c_void_p), ("kv_timestamps", ctypes.c_void_p),
        ("ts_weights", ctypes.c_void_p), ("d_ts_weights", ctypes.c_void_p),
        ("num_buckets", ctypes.c_int32), ("groups_log2", ctypes.c_int32),
    ]


class _RingTsBias(ctypes.Structure):
    _fields_ = [
        ("q_timestamps", ctypes.c_void_p), ("ts_parts", ctypes.c_void_p), ("ts_recv", ctypes.c_void_p * 2),
        ("ts_weights", ctypes.c_void_p), ("d_ts_weights", ctypes.c_void_p),
        ("num_buckets", ctypes.c_int32), ("groups_log2", ctypes.c_int32),
    ]


class _RingDesc(ctypes.Structure):
    _fields_ = [
        ("cp_size", ctypes.c_int32), ("q_rank", ctypes.c_int32), ("accumulate_dkv", ctypes.c_int32),
        ("reserved", ctypes.c_int32), ("q_rows", ctypes.c_int64), ("recv_rows", ctypes.c_int64),
        ("part_rows", ctypes.c_void_p), ("k_parts", ctypes.c_void_p), ("v_parts", ctypes.c_void_p),
        ("k_recv", ctypes.c_void_p * 2), ("v_recv", ctypes.c_void_p * 2),
        ("dk_parts", ctypes.c_void_p), ("dv_parts", ctypes.c_void_p),
    ]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads the built HIP library; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            "libhstu_attn.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`"
            " (or paper_2508_04711_amd/build.py) first; there is no fallback implementation")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32p = ctypes.c_void_p, ctypes.c_void_p
    pp = ctypes.POINTER(_Params)
    lib.hstu_jagged_attn_fwd.restype = ctypes.c_int
    lib.hstu_jagged_attn_fwd.argtypes = [pp, vp, vp, vp, i32p, vp, vp, ctypes.c_size_t, vp]
    lib.hstu_jagged_attn_fwd_static.restype = ctypes.c_int
    lib.hstu_jagged_attn_fwd_static.argtypes = [pp, vp, vp, vp, i32p, vp, vp]
    lib.hstu_static_scratch_bytes.restype = ctypes.c_size_t
    lib.hstu_static_scratch_bytes.argtypes = []
    lib.hstu_jagged_attn_bwd.restype = ctypes.c_int
    lib.hstu_jagged_attn_bwd.argtypes = [pp, vp, vp, vp, vp, i32p, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.hstu_jagged_attn_cp_partial.restype = ctypes.c_int
    lib.hstu_jagged_attn_cp_partial.argtypes = [pp, ctypes.POINTER(_CpDesc), vp, vp, vp, vp, i32p,
                                                vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.hstu_jagged_attn_workspace_bytes.restype = ctypes.c_size_t
    lib.hstu_jagged_attn_workspace_bytes.argtypes = [pp, ctypes.c_int]
    lib.hstu_validate_offsets_host.restype = ctypes.c_int
    lib.hstu_validate_offsets_host.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64]
    lib.hstu_attn_status_string.restype = ctypes.c_char_p
    lib.hstu_attn_status_string.argtypes = [ctypes.c_int]
    lib.hstu_debug_dump_schedule.restype = ctypes.c_int
    lib.hstu_debug_dump_schedule.argtypes = [pp, ctypes.POINTER(_CpDesc), ctypes.c_int, i32p,
                                             ctypes.c_void_p, ctypes.c_int32, vp, ctypes.c_size_t, vp]
    lib.hstu_debug_timing_begin.restype = ctypes.c_int
    lib.hstu_debug_timing_begin.argtypes = [ctypes.c_int]
    lib.hstu_debug_timing_end.restype = ctypes.c_int
    lib.hstu_debug_timing_end.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
    lib.hstu_cp_ring_pass.restype = ctypes.c_int
    lib.hstu_cp_ring_pass.argtypes = [pp, ctypes.POINTER(_RingDesc), vp, vp, i32p, vp, vp, vp,
                                      ctypes.c_size_t, vp, vp]
    lib.hstu_cp_ring_pass_bias.restype = ctypes.c_int
    lib.hstu_cp_ring_pass_bias.argtypes = [pp, ctypes.POINTER(_RingDesc), ctypes.POINTER(_RingTsBias), vp, vp,
                                           i32p, vp, vp, vp, ctypes.c_size_t, vp, vp]
    lib.hstu_cp_reorder.restype = ctypes.c_int
    lib.hstu_cp_reorder.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                    ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                    ctypes.c_void_p, ctypes.c_int64, i32p, vp]
    bp = ctypes.POINTER(_TsBias)
    lib.hstu_jagged_attn_bias_workspace_bytes.restype = ctypes.c_size_t
    lib.hstu_jagged_attn_bias_workspace_bytes.argtypes = [pp, ctypes.c_int]
    lib.hstu_jagged_attn_bias_fwd.restype = ctypes.c_int
    lib.hstu_jagged_attn_bias_fwd.argtypes = [pp, bp, vp, vp, vp, i32p, vp, vp, ctypes.c_size_t, vp]
    lib.hstu_jagged_attn_bias_bwd.restype = ctypes.c_int
    lib.hstu_jagged_attn_bias_bwd.argtypes = [pp, bp, vp, vp, vp, vp, i32p, vp, vp, vp, vp,
                                              ctypes.c_size_t, vp]
    lib.hstu_jagged_attn_cp_partial_bias.restype = ctypes.c_int
    lib.hstu_jagged_attn_cp_partial_bias.argtypes = [pp, ctypes.POINTER(_CpDesc), ctypes.POINTER(_CpTsBias),
                                                     vp, vp, vp, vp, i32p, vp, vp, vp, vp, vp,
                                                     ctypes.c_size_t, vp]
    lib.hstu_debug_mfma_loop.restype = ctypes.c_int
    lib.hstu_debug_mfma_loop.argtypes = [ctypes.c_int, ctypes.c_int, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.hstu_debug_dq_atomic_rate.restype = ctypes.c_int
    lib.hstu_debug_dq_atomic_rate.argtypes = [vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                              ctypes.POINTER(ctypes.c_double), vp]
    lib.hstu_schedule_tile_rows.restype = ctypes.c_int
    lib.hstu_schedule_tile_rows.argtypes = [pp, ctypes.c_int]
    _lib = lib
    return lib


def hstu_attn_status_string(status: int) -> str:
    return load_library().hstu_attn_status_string(int(status)).decode()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return HSTU_BF16
    if t.dtype == torch.float32:
        return HSTU_F32
    raise TypeError("unsupported dtype %s" % t.dtype)


def _params(batch, num_heads, d_qk, d_v, max_len, alpha, causal, dtype_code, total_rows,
            out_dtype_code=None) -> _Params:
    return _Params(int(batch), int(num_heads), int(d_qk), int(d_v), int(max_len), float(alpha),
                   int(bool(causal)), int(dtype_code), int(total_rows),
                   int(dtype_code if out_dtype_code is None else out_dtype_code), int(default_flags))


def _out_dtype(in_dtype: torch.dtype, out_dtype: Optional[torch.dtype]) -> torch.dtype:
    return in_dtype if out_dtype is None else out_dtype


def _code(dt: torch.dtype) -> int:
    if dt == torch.bfloat16:
        return HSTU_BF16
    if dt == torch.float32:
        return HSTU_F32
    raise TypeError("unsupported dtype %s" % dt)


def _ptr(t: Optional[torch.Tensor]):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _allocates_on_its_stream(fn):
    """Runs `fn` with its `stream=` argument as torch's current stream, so that whatever the function
    allocates (outputs, workspace) belongs to the stream its kernels are queued on: the caching
    allocator then cannot hand that memory to another stream's allocation while they still run."""
    @functools.wraps(fn)
    def wrapped(*args, **kwargs):
        stream = kwargs.get("stream")
        if stream is None or stream == torch.cuda.current_stream():
            return fn(*args, **kwargs)
        with torch.cuda.stream(stream):
            return fn(*args, **kwargs)
    return wrapped


def _check_tensor(t: torch.Tensor, name: str, rows: int, heads: int, dim: int, dtype) -> None:
    if not t.is_cuda:
        raise ValueError("%s must be a device tensor" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if tuple(t.shape) != (rows, heads, dim) or t.dtype != dtype:
        raise ValueError("%s: expected %s %s, got %s %s" % (name, (rows, heads, dim), dtype,
                                                          tuple(t.shape), t.dtype))


def _workspace(params: _Params, which: int, workspace: Optional[torch.Tensor], device) -> torch.Tensor:
    need = hstu_jagged_attn_workspace_bytes(params, which)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    return workspace


def hstu_jagged_attn_workspace_bytes(params_or_tuple, which: int) -> int:
    """Bytes of device workspace the entry point `which` (0 fwd, 1 bwd, 2 cp) needs."""
    p = params_or_tuple if isinstance(params_or_tuple, _Params) else _params(*params_or_tuple)
    return int(load_library().hstu_jagged_attn_workspace_bytes(ctypes.byref(p), int(which)))


def hstu_validate_offsets_host(host_offsets, total_rows: int) -> int:
    off = np.ascontiguousarray(host_offsets, dtype=np.int32)
    return int(load_library().hstu_validate_offsets_host(
        off.ctypes.data_as(ctypes.c_void_p), len(off) - 1, int(total_rows)))


@_allocates_on_its_stream
def hstu_jagged_attn_fwd(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                         seq_offsets: torch.Tensor, max_len: int, alpha: float, causal: bool = True,
                         out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                         stream=None, out_dtype: Optional[torch.dtype] = None) -> torch.Tensor:
    """O = Mask(SiLU(alpha Q K^T)) V / max_len over a jagged batch; q,k: [T,H,d_qk], v: [T,H,d_v].

    out_dtype: dtype of the result (default: the inputs'; torch.float32 keeps the accumulators).
    """
    T, H, dqk = q.shape
    dv = v.shape[2]
    _check_tensor(q, "q", T, H, dqk, q.dtype); _check_tensor(k, "k", T, H, dqk, q.dtype)
    _check_tensor(v, "v", T, H, dv, q.dtype)
    if seq_offsets.dtype != torch.int32 or not seq_offsets.is_cuda or not seq_offsets.is_contiguous():
        raise ValueError("seq_offsets must be a contiguous int32 device tensor")
    B = seq_offsets.numel() - 1
    odt = out.dtype if out is not None else _out_dtype(q.dtype, out_dtype)
    if out is None:
        out = torch.empty((T, H, dv), dtype=odt, device=q.device)
    else:
        _check_tensor(out, "out", T, H, dv, odt)
    p = _params(B, H, dqk, dv, max_len, alpha, causal, _dtype_code(q), T, _code(odt))
    ws = _workspace(p, HSTU_WS_FWD, workspace, q.device)
    rc = load_library().hstu_jagged_attn_fwd(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v),
                                             _ptr(seq_offsets), _ptr(out), _ptr(ws), ws.numel(),
                                             _stream(stream))
    if rc != 0:
        raise HstuError(rc, "hstu_jagged_attn_fwd")
    return out


def hstu_static_scratch_bytes() -> int:
    """Size of the static device array hstu_jagged_attn_fwd_static works in."""
    return int(load_library().hstu_static_scratch_bytes())


def hstu_jagged_attn_fwd_static(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                                seq_offsets: torch.Tensor, max_len: int, alpha: float,
                                causal: bool, out: torch.Tensor, stream=None) -> torch.Tensor:
    """hstu_jagged_attn_fwd without a workspace and without any allocation: `out` is the caller's."""
    T, H, dqk = q.shape
    dv = v.shape[2]
    _check_tensor(q, "q", T, H, dqk, q.dtype); _check_tensor(k, "k", T, H, dqk, q.dtype)
    _check_tensor(v, "v", T, H, dv, q.dtype); _check_tensor(out, "out", T, H, dv, out.dtype)
    if seq_offsets.dtype != torch.int32 or not seq_offsets.is_cuda or not seq_offsets.is_contiguous():
        raise ValueError("seq_offsets must be a contiguous int32 device tensor")
    p = _params(seq_offsets.numel() - 1, H, dqk, dv, max_len, alpha, causal, _dtype_code(q), T,
                _code(out.dtype))
    rc = load_library().hstu_jagged_attn_fwd_static(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v),
                                                    _ptr(seq_offsets), _ptr(out), _stream(stream))
    if rc != 0:
        raise HstuError(rc, "hstu_jagged_attn_fwd_static")
    return out


@_allocates_on_its_stream
def hstu_jagged_attn_bwd(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, d_o: torch.Tensor,
                         seq_offsets: torch.Tensor, max_len: int, alpha: float, causal: bool = True,
                         out: Optional[Tuple[torch.Tensor, torch.Tensor, torch.Tensor]] = None,
                         workspace: Optional[torch.Tensor] = None, stream=None,
                         out_dtype: Optional[torch.dtype] = None
                         ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """(dQ, dK, dV) of sum(O * d_o) for the forward above."""
    T, H, dqk = q.shape
    dv = v.shape[2]
    _check_tensor(q, "q", T, H, dqk, q.dtype); _check_tensor(k, "k", T, H, dqk, q.dtype)
    _check_tensor(v, "v", T, H, dv, q.dtype); _check_tensor(d_o, "d_o", T, H, dv, q.dtype)
    if seq_offsets.dtype != torch.int32 or not seq_offsets.is_cuda or not seq_offsets.is_contiguous():
        raise ValueError("seq_offsets must be a contiguous int32 device tensor")
    B = seq_offsets.numel() - 1
    odt = out[0].dtype if out is not None else _out_dtype(q.dtype, out_dtype)
    if out is None:
        dq = torch.empty_like(q, dtype=odt); dk = torch.empty_like(k, dtype=odt)
        dvv = torch.empty_like(v, dtype=odt)
    else:
        dq, dk, dvv = out
        _check_tensor(dq, "dq", T, H, dqk, odt); _check_tensor(dk, "dk", T, H, dqk, odt)
        _check_tensor(dvv, "dv", T, H, dv, odt)
    p = _params(B, H, dqk, dv, max_len, alpha, causal, _dtype_code(q), T, _code(odt))
    ws = _workspace(p, HSTU_WS_BWD, workspace, q.device)
    rc = load_library().hstu_jagged_attn_bwd(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(d_o),
                                             _ptr(seq_offsets), _ptr(dq), _ptr(dk), _ptr(dvv),
                                             _ptr(ws), ws.numel(), _stream(stream))
    if rc != 0:
        raise HstuError(rc, "hstu_jagged_attn_bwd")
    return dq, dk, dvv


def hstu_jagged_attn_bias_workspace_bytes(params_or_tuple, which: int) -> int:
    """Bytes of device workspace of the calls with timestamp bias (`which`: 0 fwd, 1 bwd)."""
    p = params_or_tuple if isinstance(params_or_tuple, _Params) else _params(*params_or_tuple)
    return int(load_library().hstu_jagged_attn_bias_workspace_bytes(ctypes.byref(p), int(which)))


def _bias_desc(timestamps, ts_weights, d_ts_weights, groups_log2, rows) -> _TsBias:
    if timestamps.dtype != torch.int32 or not timestamps.is_cuda or not timestamps.is_contiguous() \
            or tuple(timestamps.shape) != (rows,):
        raise ValueError("timestamps must be a contiguous int32 device tensor of one entry per row")
    for name, t in (("ts_weights", ts_weights), ("d_ts_weights", d_ts_weights)):
        if t is None:
            continue
        if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous() or t.dim() != 1:
            raise ValueError("%s must be a contiguous 1-d fp32 device tensor" % name)
    if d_ts_weights is not None and d_ts_weights.numel() != ts_weights.numel():
        raise ValueError("d_ts_weights must have one entry per bucket")
    return _TsBias(timestamps.data_ptr(), ts_weights.data_ptr(),
                   d_ts_weights.data_ptr() if d_ts_weights is not None else None,
                   int(ts_weights.numel()), int(groups_log2))


def _bias_workspace(params: _Params, which: int, workspace, device) -> torch.Tensor:
    if workspace is None:
        need = hstu_jagged_attn_bias_workspace_bytes(params, which)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    return workspace


@_allocates_on_its_stream
def hstu_jagged_attn_bias_fwd(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                              seq_offsets: torch.Tensor, timestamps: torch.Tensor,
                              ts_weights: torch.Tensor, groups_log2: int, max_len: int, alpha: float,
                              causal: bool = True, out: Optional[torch.Tensor] = None,
                              workspace: Optional[torch.Tensor] = None, stream=None,
                              out_dtype: Optional[torch.dtype] = None) -> torch.Tensor:
    """hstu_jagged_attn_fwd with the timestamp bias: x = alpha * (q.k + ts_weights[bucket])."""
    T, H, dqk = q.shape
    dv = v.shape[2]
    _check_tensor(q, "q", T, H, dqk, q.dtype); _check_tensor(k, "k", T, H, dqk, q.dtype)
    _check_tensor(v, "v", T, H, dv, q.dtype)
    if seq_offsets.dtype != torch.int32 or not seq_offsets.is_cuda or not seq_offsets.is_contiguous():
        raise ValueError("seq_offsets must be a contiguous int32 device tensor")
    B = seq_offsets.numel() - 1
    odt = out.dtype if out is not None else _out_dtype(q.dtype, out_dtype)
    if out is None:
        out = torch.empty((T, H, dv), dtype=odt, device=q.device)
    else:
        _check_tensor(out, "out", T, H, dv, odt)
    p = _params(B, H, dqk, dv, max_len, alpha, causal, _dtype_code(q), T, _code(odt))
    bias = _bias_desc(timestamps, ts_weights, None, groups_log2, T)
    ws = _bias_workspace(p, HSTU_WS_FWD, workspace, q.device)
    rc = load_library().hstu_jagged_attn_bias_fwd(ctypes.byref(p), ctypes.byref(bias), _ptr(q), _ptr(k),
                                                  _ptr(v), _ptr(seq_offsets), _ptr(out), _ptr(ws),
                                                  ws.numel(), _stream(stream))
    if rc != 0:
        raise HstuError(rc, "hstu_jagged_attn_bias_fwd")
    return out


@_allocates_on_its_stream
def hstu_jagged_attn_bias_bwd(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, d_o: torch.Tensor,
                              seq_offsets: torch.Tensor, timestamps: torch.Tensor,
                              ts_weights: torch.Tensor, groups_log2: int, max_len: int, alpha: float,
                              causal: bool = True, out: Optional[tuple] = None,
                              workspace: Optional[torch.Tensor] = None, stream=None,
                              out_dtype: Optional[torch.dtype] = None):
    """(dQ, dK, dV, d_ts_weights) of sum(O * d_o) for the forward with bias; `out` may pass the four."""
    T, H, dqk = q.shape
    dv = v.shape[2]
    _check_tensor(q, "q", T, H, dqk, q.dtype); _check_tensor(k, "k", T, H, dqk, q.dtype)
    _check_tensor(v, "v", T, H, dv, q.dtype); _check_tensor(d_o, "d_o", T, H, dv, q.dtype)
    if seq_offsets.dtype != torch.int32 or not seq_offsets.is_cuda or not seq_offsets.is_contiguous():
        raise ValueError("seq_offsets must be a contiguous int32 device tensor")
    B = seq_offsets.numel() - 1
    odt = out[0].dtype if out is not None else _out_dtype(q.dtype, out_dtype)
    if out is None:
        dq = torch.empty_like(q, dtype=odt); dk = torch.empty_like(k, dtype=odt)
        dvv = torch.empty_like(v, dtype=odt)
        dw = torch.empty_like(ts_weights)
    else:
        dq, dk, dvv, dw = out
        _check_tensor(dq, "dq", T, H, dqk, odt); _check_tensor(dk, "dk", T, H, dqk, odt)
        _check_tensor(dvv, "dv", T, H, dv, odt)
    p = _params(B, H, dqk, dv, max_len, alpha, causal, _dtype_code(q), T, _code(odt))
    bias = _bias_desc(timestamps, ts_weights, dw, groups_log2, T)
    ws = _bias_workspace(p, HSTU_WS_BWD, workspace, q.device)
    rc = load_library().hstu_jagged_attn_bias_bwd(ctypes.byref(p), ctypes.byref(bias), _ptr(q), _ptr(k),
                                                  _ptr(v), _ptr(d_o), _ptr(seq_offsets), _ptr(dq),
                                                  _ptr(dk), _ptr(dvv), _ptr(ws), ws.numel(),
                                                  _stream(stream))
    if rc != 0:
        raise HstuError(rc, "hstu_jagged_attn_bias_bwd")
    return dq, dk, dvv, dw


@_allocates_on_its_stream
def hstu_jagged_attn_cp_partial(q_local: torch.Tensor, k_part: torch.Tensor, v_part: torch.Tensor,
                                d_o_local: Optional[torch.Tensor], seq_offsets_global: torch.Tensor,
                                total_rows: int, max_len: int, alpha: float, causal: bool,
                                cp_size: int, q_rank: int, kv_rank: int, accumulate: bool = False,
                                out: Optional[tuple] = None, want_o: bool = True,
                                workspace: Optional[torch.Tensor] = None, stream=None,
                                out_dtype: Optional[torch.dtype] = None):
    """One context-parallel rank's partial: returns (o_local, dq_local, dk_part, dv_part).

    The gradients are None when d_o_local is None; o_local is None when want_o is False.
    `out` may pass the four output tensors (required when accumulate is set).
    """
    nq, H, dqk = q_local.shape
    nk, _, dv = v_part.shape
    dt = q_local.dtype
    _check_tensor(q_local, "q_local", nq, H, dqk, dt); _check_tensor(k_part, "k_part", nk, H, dqk, dt)
    _check_tensor(v_part, "v_part", nk, H, dv, dt)
    if d_o_local is not None:
        _check_tensor(d_o_local, "d_o_local", nq, H, dv, dt)
    so = seq_offsets_global
    if so.dtype != torch.int32 or not so.is_cuda or not so.is_contiguous():
        raise ValueError("seq_offsets_global must be a contiguous int32 device tensor")
    B = so.numel() - 1
    odt = _out_dtype(dt, out_dtype)
    if out is not None:
        o, dq, dk, dvv = out
        first = next(t for t in out if t is not None)
        odt = first.dtype
        for t, name, rows, dim in ((o, "o_local", nq, dv), (dq, "dq_local", nq, dqk),
                                   (dk, "dk_part", nk, dqk), (dvv, "dv_part", nk, dv)):
            if t is not None:
                _check_tensor(t, name, rows, H, dim, odt)
    else:
        if accumulate:
            raise ValueError("accumulate needs the outputs to add to")
        o = torch.empty((nq, H, dv), dtype=odt, device=q_local.device) if want_o else None
        if d_o_local is not None:
            dq = torch.empty_like(q_local, dtype=odt); dk = torch.empty_like(k_part, dtype=odt)
            dvv = torch.empty_like(v_part, dtype=odt)
        else:
            dq = dk = dvv = None
    p = _params(B, H, dqk, dv, max_len, alpha, causal, _dtype_code(q_local), total_rows, _code(odt))
    desc = _CpDesc(int(cp_size), int(q_rank), int(kv_rank), int(bool(accumulate)), int(nq), int(nk))
    ws = _workspace(p, HSTU_WS_CP, workspace, q_local.device)
    rc = load_library().hstu_jagged_attn_cp_partial(
        ctypes.byref(p), ctypes.byref(desc), _ptr(q_local), _ptr(k_part), _ptr(v_part),
        _ptr(d_o_local), _ptr(so), _ptr(o), _ptr(dq), _ptr(dk), _ptr(dvv), _ptr(ws), ws.numel(),
        _stream(stream))
    if rc != 0:
        raise HstuError(rc, "hstu_jagged_attn_cp_partial")
    return o, dq, dk, dvv


@_allocates_on_its_stream
def hstu_jagged_attn_cp_partial_bias(q_local: torch.Tensor, k_part: torch.Tensor, v_part: torch.Tensor,
                                     d_o_local: Optional[torch.Tensor], seq_offsets_global: torch.Tensor,
                                     total_rows: int, q_timestamps: torch.Tensor,
                                     kv_timestamps: torch.Tensor, ts_weights: torch.Tensor,
                                     groups_log2: int, max_len: int, alpha: float, causal: bool,
                                     cp_size: int, q_rank: int, kv_rank: int, accumulate: bool = False,
                                     out: Optional[tuple] = None, want_o: bool = True,
                                     workspace: Optional[torch.Tensor] = None, stream=None,
                                     out_dtype: Optional[torch.dtype] = None):
    """hstu_jagged_attn_cp_partial with the timestamp bias: returns (o_local, dq_local, dk_part,
    dv_part, d_ts_weights); the timestamps are those of the rows of q_local and of k_part.
    `out` may pass the five output tensors (required when accumulate is set)."""
    nq, H, dqk = q_local.shape
    nk, _, dv = v_part.shape
    dt = q_local.dtype
    _check_tensor(q_local, "q_local", nq, H, dqk, dt); _check_tensor(k_part, "k_part", nk, H, dqk, dt)
    _check_tensor(v_part, "v_part", nk, H, dv, dt)
    if d_o_local is not None:
        _check_tensor(d_o_local, "d_o_local", nq, H, dv, dt)
    so = seq_offsets_global
    if so.dtype != torch.int32 or not so.is_cuda or not so.is_contiguous():
        raise ValueError("seq_offsets_global must be a contiguous int32 device tensor")
    B = so.numel() - 1
    odt = _out_dtype(dt, out_dtype)
    if out is not None:
        o, dq, dk, dvv, dw = out
        first = next(t for t in out[:4] if t is not None)
        odt = first.dtype
        for t, name, rows, dim in ((o, "o_local", nq, dv), (dq, "dq_local", nq, dqk),
                                   (dk, "dk_part", nk, dqk), (dvv, "dv_part", nk, dv)):
            if t is not None:
                _check_tensor(t, name, rows, H, dim, odt)
    else:
        if accumulate:
            raise ValueError("accumulate needs the outputs to add to")
        o = torch.empty((nq, H, dv), dtype=odt, device=q_local.device) if want_o else None
        if d_o_local is not None:
            dq = torch.empty_like(q_local, dtype=odt); dk = torch.empty_like(k_part, dtype=odt)
            dvv = torch.empty_like(v_part, dtype=odt)
            dw = torch.empty_like(ts_weights)
        else:
            dq = dk = dvv = dw = None
    for name, t, rows in (("q_timestamps", q_timestamps, nq), ("kv_timestamps", kv_timestamps, nk)):
        if t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != (rows,):
            raise ValueError("%s must be a contiguous int32 device tensor of one entry per row" % name)
    for name, t in (("ts_weights", ts_weights), ("d_ts_weights", dw)):
        if t is not None and (t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous()
                              or t.dim() != 1 or t.numel() != ts_weights.numel()):
            raise ValueError("%s must be a contiguous 1-d fp32 device tensor of one entry per bucket" % name)
    p = _params(B, H, dqk, dv, max_len, alpha, causal, _dtype_code(q_local), total_rows, _code(odt))
    desc = _CpDesc(int(cp_size), int(q_rank), int(kv_rank), int(bool(accumulate)), int(nq), int(nk))
    bias = _CpTsBias(q_timestamps.data_ptr(), kv_timestamps.data_ptr(), ts_weights.data_ptr(),
                     dw.data_ptr() if dw is not None else None, int(ts_weights.numel()), int(groups_log2))
    ws = _bias_workspace(p, HSTU_WS_CP, workspace, q_local.device)
    rc = load_library().hstu_jagged_attn_cp_partial_bias(
        ctypes.byref(p), ctypes.byref(desc), ctypes.byref(bias), _ptr(q_local), _ptr(k_part), _ptr(v_part),
        _ptr(d_o_local), _ptr(so), _ptr(o), _ptr(dq), _ptr(dk), _ptr(dvv), _ptr(ws), ws.numel(),
        _stream(stream))
    if rc != 0:
        raise HstuError(rc, "hstu_jagged_attn_cp_partial_bias")
    return o, dq, dk, dvv, dw


def hstu_schedule_tile_rows(dtype_code: int, d_qk: int, d_v: int, side: int, total_rows: int = 1,
                            num_heads: int = 1, batch: int = 1) -> int:
    """Owner rows per schedule item on `side` for a whole-batch problem of the given size."""
    p = _params(batch, num_heads, d_qk, d_v, 1, 1.0, True, dtype_code, total_rows)
    return int(load_library().hstu_schedule_tile_rows(ctypes.byref(p), int(side)))


@_allocates_on_its_stream
def hstu_debug_dump_schedule(seq_offsets: torch.Tensor, total_rows: int, num_heads: int, d_qk: int,
                             d_v: int, causal: bool, dtype_code: int, side: int,
                             cp: Optional[Tuple[int, int, int, int, int]] = None,
                             max_len: int = 1, workspace: Optional[torch.Tensor] = None) -> np.ndarray:
    """The device-built schedule as an int32 array [n_items, 12] in schedule order.

    cp = (cp_size, q_rank, kv_rank, q_rows, kv_rows) for a context-parallel problem.  The last
    column is 0, or p > 0 for an item that covers a part of its tile's keys (partial slot p - 1).
    """
    B = seq_offsets.numel() - 1
    p = _params(B, num_heads, d_qk, d_v, max_len, 1.0, causal, dtype_code, total_rows)
    desc = None
    if cp is not None:
        desc = _CpDesc(int(cp[0]), int(cp[1]), int(cp[2]), 0, int(cp[3]), int(cp[4]))
    ws = _workspace(p, HSTU_WS_CP if cp is not None else HSTU_WS_FWD, workspace, seq_offsets.device)
    max_items = int(total_rows) // 32 + 2 * B + 8 + 2048
    buf = np.zeros((max_items, 12), dtype=np.int32)
    n = load_library().hstu_debug_dump_schedule(
        ctypes.byref(p), ctypes.byref(desc) if desc is not None else None, int(side),
        _ptr(seq_offsets), buf.ctypes.data_as(ctypes.c_void_p), max_items, _ptr(ws), ws.numel(),
        _stream(None))
    if n < 0:
        raise HstuError(n, "hstu_debug_dump_schedule")
    return buf[:n].copy()


KERNEL_KINDS = {0: "fwd", 1: "dkdv", 2: "dq", 3: "plan", 4: "transpose", 5: "reorder", 6: "reduce",
                7: "ts_records", 8: "dw_finish", 9: "mfma_loop", 10: "dq_atomic"}


def hstu_debug_mfma_loop(random_operands: bool, iterations: int, sink: torch.Tensor, stream=None) -> float:
    """Queues one launch of the matrix-instruction loop; returns its flops (the caller times it)."""
    flops = ctypes.c_double(0.0)
    rc = load_library().hstu_debug_mfma_loop(int(bool(random_operands)), int(iterations), _ptr(sink),
                                             ctypes.byref(flops), _stream(stream))
    if rc != 0:
        raise HstuError(rc, "hstu_debug_mfma_loop")
    return flops.value


def hstu_debug_dq_atomic_rate(dq_f32: torch.Tensor, blocks: int, head_per_xcd: bool, stream=None) -> float:
    """Queues one launch of the atomic-rate kernel on dq_f32 [rows, heads, 128] fp32; returns the
    bytes it adds (the caller times it)."""
    rows, heads, d = dq_f32.shape
    if d != 128 or dq_f32.dtype != torch.float32 or not dq_f32.is_contiguous() or not dq_f32.is_cuda:
        raise ValueError("dq_f32 must be a contiguous fp32 device tensor [rows, heads, 128]")
    nbytes = ctypes.c_double(0.0)
    rc = load_library().hstu_debug_dq_atomic_rate(_ptr(dq_f32), int(rows), int(heads), int(blocks),
                                                  int(bool(head_per_xcd)), ctypes.byref(nbytes), _stream(stream))
    if rc != 0:
        raise HstuError(rc, "hstu_debug_dq_atomic_rate")
    return nbytes.value


def hstu_debug_timing_begin(max_records: int = 4096) -> None:
    rc = load_library().hstu_debug_timing_begin(int(max_records))
    if rc != 0:
        raise HstuError(rc, "hstu_debug_timing_begin")


def hstu_debug_timing_end(capacity: int = 4096):
    """List of (kind name, milliseconds), one per kernel launched since timing began."""
    kinds = np.zeros(capacity, dtype=np.int32)
    ms = np.zeros(capacity, dtype=np.float32)
    n = load_library().hstu_debug_timing_end(kinds.ctypes.data_as(ctypes.c_void_p),
                                             ms.ctypes.data_as(ctypes.c_void_p), int(capacity))
    if n < 0:
        raise HstuError(n, "hstu_debug_timing_end")
    return [(KERNEL_KINDS.get(int(kinds[i]), "?"), float(ms[i])) for i in range(n)]


@_allocates_on_its_stream
def hstu_cp_reorder(tensors, seq_offsets: torch.Tensor, total_rows: int, cp_size: int, rank: int,
                    local_rows: int, scatter: bool = False, out=None, stream=None):
    """Moves rows between the global jagged layout and `rank`'s local layout (up to 4 tensors).

    gather (scatter=False): tensors are global [total_rows, ...]; returns local [local_rows, ...].
    scatter=True: tensors are local; `out` must give the global tensors to write the rank's rows into.
    """
    tensors = list(tensors)
    n = len(tensors)
    if not 1 <= n <= 4:
        raise ValueError("1 to 4 tensors per call")
    rows_in = local_rows if scatter else total_rows
    rows_out = total_rows if scatter else local_rows
    for t in tensors:
        if not t.is_cuda or not t.is_contiguous() or t.shape[0] != rows_in:
            raise ValueError("tensors must be contiguous device tensors with %d rows" % rows_in)
    if out is None:
        if scatter:
            raise ValueError("scatter needs the global tensors to write into")
        out = [torch.empty((rows_out,) + tuple(t.shape[1:]), dtype=t.dtype, device=t.device) for t in tensors]
    out = list(out)
    for t, o in zip(tensors, out):
        if (not o.is_cuda or not o.is_contiguous() or o.shape[0] != rows_out or o.dtype != t.dtype
                or tuple(o.shape[1:]) != tuple(t.shape[1:])):
            raise ValueError("output tensors must match the inputs in dtype and row shape")
    B = seq_offsets.numel() - 1
    lib = load_library()
    src = (ctypes.c_void_p * n)(*[t.data_ptr() for t in tensors])
    dst = (ctypes.c_void_p * n)(*[o.data_ptr() for o in out])
    rb = (ctypes.c_int64 * n)(*[int(np.prod(t.shape[1:], dtype=np.int64)) * t.element_size()
                                for t in tensors])
    rc = lib.hstu_cp_reorder(B, int(total_rows), int(cp_size), int(rank), int(bool(scatter)), n,
                             ctypes.cast(src, ctypes.c_void_p), ctypes.cast(dst, ctypes.c_void_p),
                             ctypes.cast(rb, ctypes.c_void_p), int(local_rows), _ptr(seq_offsets),
                             _stream(stream))
    if rc != 0:
        raise HstuError(rc, "hstu_cp_reorder")
    return out


_copy_streams = {}


def hstu_cp_ring_pass(q_local: torch.Tensor, d_o_local: Optional[torch.Tensor], k_parts, v_parts,
                      seq_offsets_global: torch.Tensor, total_rows: int, max_len: int, alpha: float,
                      causal: bool, cp_size: int, q_rank: int, out_dtype: torch.dtype = torch.float32,
                      accumulate_dkv: bool = False, out: Optional[tuple] = None, recv=None,
                      workspace: Optional[torch.Tensor] = None, stream=None, copy_stream=None,
                      _bias=None):
    """One rank's context-parallel pass as a ring over the K/V parts of all ranks.

    k_parts / v_parts: one tensor per rank (its rows of K and V in its local layout), standing
    for the peers' memory.  Returns (o_local, dq_local, dk_parts, dv_parts); the gradients are
    None when d_o_local is None.  `out` may pass them (needed when accumulate_dkv is set), `recv`
    the four receive buffers (k0, k1, v0, v1).
    """
    nq, H, dqk = q_local.shape
    dv = v_parts[0].shape[2]
    dt = q_local.dtype
    dev = q_local.device
    if len(k_parts) != cp_size or len(v_parts) != cp_size:
        raise ValueError("one K part and one V part per rank")
    _check_tensor(q_local, "q_local", nq, H, dqk, dt)
    if d_o_local is not None:
        _check_tensor(d_o_local, "d_o_local", nq, H, dv, dt)
    rows = [int(k.shape[0]) for k in k_parts]
    for r in range(cp_size):
        _check_tensor(k_parts[r], "k_parts[%d]" % r, rows[r], H, dqk, dt)
        _check_tensor(v_parts[r], "v_parts[%d]" % r, rows[r], H, dv, dt)
    so = seq_offsets_global
    if so.dtype != torch.int32 or not so.is_cuda or not so.is_contiguous():
        raise ValueError("seq_offsets_global must be a contiguous int32 device tensor")
    backward = d_o_local is not None
    if out is not None:
        o, dq, dks, dvs = out
        out_dtype = next(t for t in (o, dq) if t is not None).dtype
    else:
        if accumulate_dkv:
            raise ValueError("accumulate_dkv needs the key-side gradients to add to")
        o = torch.empty((nq, H, dv), dtype=out_dtype, device=dev)
        dq = torch.empty((nq, H, dqk), dtype=out_dtype, device=dev) if backward else None
        dks = [torch.empty((rows[r], H, dqk), dtype=out_dtype, device=dev) for r in range(cp_size)] if backward else None
        dvs = [torch.empty((rows[r], H, dv), dtype=out_dtype, device=dev) for r in range(cp_size)] if backward else None
    if o is not None:
        _check_tensor(o, "o_local", nq, H, dv, out_dtype)
    if backward:
        _check_tensor(dq, "dq_local", nq, H, dqk, out_dtype)
        for r in range(cp_size):
            _check_tensor(dks[r], "dk_parts[%d]" % r, rows[r], H, dqk, out_dtype)
            _check_tensor(dvs[r], "dv_parts[%d]" % r, rows[r], H, dv, out_dtype)
    recv_rows = max([rows[r] for r in range(cp_size) if r != q_rank] + [0])
    if recv is None:
        recv = [torch.empty((max(recv_rows, 1), H, d), dtype=dt, device=dev) for d in (dqk, dqk, dv, dv)]
    else:
        recv_rows = min(int(t.shape[0]) for t in recv)
    if stream is None:
        stream = torch.cuda.current_stream()
    if copy_stream is None:
        key = (dev.index, stream.cuda_stream)
        if key not in _copy_streams:
            _copy_streams[key] = torch.cuda.Stream(device=dev)  # default priority
        copy_stream = _copy_streams[key]
    p = _params(so.numel() - 1, H, dqk, dv, max_len, alpha, causal, _dtype_code(q_local), total_rows,
                _code(out_dtype))
    arr = lambda ts: (ctypes.c_void_p * cp_size)(*[t.data_ptr() if t is not None and t.numel() else None for t in ts])
    part_rows = (ctypes.c_int64 * cp_size)(*rows)
    kp, vp_ = arr(k_parts), arr(v_parts)
    dkp = arr(dks) if backward else None
    dvp = arr(dvs) if backward else None
    desc = _RingDesc(int(cp_size), int(q_rank), int(bool(accumulate_dkv)), 0, int(nq), int(recv_rows),
                     ctypes.cast(part_rows, ctypes.c_void_p), ctypes.cast(kp, ctypes.c_void_p),
                     ctypes.cast(vp_, ctypes.c_void_p),
                     (ctypes.c_void_p * 2)(recv[0].data_ptr(), recv[1].data_ptr()),
                     (ctypes.c_void_p * 2)(recv[2].data_ptr(), recv[3].data_ptr()),
                     ctypes.cast(dkp, ctypes.c_void_p) if backward else None,
                     ctypes.cast(dvp, ctypes.c_void_p) if backward else None)
    if _bias is not None:
        q_ts, ts_parts, ts_weights, groups_log2, dw = _bias
        if len(ts_parts) != cp_size:
            raise ValueError("one timestamp tensor per rank")
        for name, t, n in [("q_timestamps", q_ts, nq)] + [("ts_parts[%d]" % r, ts_parts[r], rows[r])
                                                         for r in range(cp_size)]:
            if t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != (n,):
                raise ValueError("%s must be a contiguous int32 device tensor of one entry per row" % name)
        if backward and dw is None:
            dw = torch.empty_like(ts_weights)
        ts_recv = [torch.empty(max(recv_rows, 1), dtype=torch.int32, device=dev) for _ in range(2)]
        tsp = arr(ts_parts)
        bias = _RingTsBias(q_ts.data_ptr(), ctypes.cast(tsp, ctypes.c_void_p),
                           (ctypes.c_void_p * 2)(ts_recv[0].data_ptr(), ts_recv[1].data_ptr()),
                           ts_weights.data_ptr(), dw.data_ptr() if dw is not None else None,
                           int(ts_weights.numel()), int(groups_log2))
        ws = _bias_workspace(p, HSTU_WS_CP, workspace, dev)
        rc = load_library().hstu_cp_ring_pass_bias(
            ctypes.byref(p), ctypes.byref(desc), ctypes.byref(bias), _ptr(q_local), _ptr(d_o_local), _ptr(so),
            _ptr(o), _ptr(dq), _ptr(ws), ws.numel(), ctypes.c_void_p(stream.cuda_stream),
            ctypes.c_void_p(copy_stream.cuda_stream))
        if rc != 0:
            raise HstuError(rc, "hstu_cp_ring_pass_bias")
        for t in list(recv) + list(k_parts) + list(v_parts) + ts_recv + list(ts_parts):
            t.record_stream(copy_stream)
        return o, dq, dks, dvs, dw
    ws = _workspace(p, HSTU_WS_CP, workspace, dev)
    rc = load_library().hstu_cp_ring_pass(
        ctypes.byref(p), ctypes.byref(desc), _ptr(q_local), _ptr(d_o_local), _ptr(so), _ptr(o), _ptr(dq),
        _ptr(ws), ws.numel(), ctypes.c_void_p(stream.cuda_stream), ctypes.c_void_p(copy_stream.cuda_stream))
    if rc != 0:
        raise HstuError(rc, "hstu_cp_ring_pass")
    # the receive buffers and the parts are read by work still in flight on the copy stream
    for t in list(recv) + list(k_parts) + list(v_parts):
        t.record_stream(copy_stream)
    return o, dq, dks, dvs


def hstu_cp_ring_pass_bias(q_local: torch.Tensor, d_o_local: Optional[torch.Tensor], k_parts, v_parts,
                           seq_offsets_global: torch.Tensor, total_rows: int, q_timestamps: torch.Tensor,
                           ts_parts, ts_weights: torch.Tensor, groups_log2: int, max_len: int, alpha: float,
                           causal: bool, cp_size: int, q_rank: int, out_dtype: torch.dtype = torch.float32,
                           accumulate_dkv: bool = False, out: Optional[tuple] = None, recv=None,
                           workspace: Optional[torch.Tensor] = None, stream=None, copy_stream=None):
    """hstu_cp_ring_pass with the timestamp bias: ts_parts[r] holds the timestamps of rank r's rows,
    q_timestamps those of q_local.  Returns (o_local, dq_local, dk_parts, dv_parts, d_ts_weights);
    `out` may pass the five (d_ts_weights is overwritten with the rank's sum over its steps)."""
    dw = None
    if out is not None:
        out, dw = tuple(out[:4]), out[4]
    return hstu_cp_ring_pass(q_local, d_o_local, k_parts, v_parts, seq_offsets_global, total_rows, max_len,
                             alpha, causal, cp_size, q_rank, out_dtype=out_dtype,
                             accumulate_dkv=accumulate_dkv, out=out, recv=recv, workspace=workspace,
                             stream=stream, copy_stream=copy_stream,
                             _bias=(q_timestamps, ts_parts, ts_weights, groups_log2, dw))

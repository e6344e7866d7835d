"""CPU oracle for jagged HSTU attention -- TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It shares no code with the GPU library and never imports it.

`hstu_oracle.c` holds the arithmetic (double precision, one (query, key) pair
at a time, straight from the HSTU attention equation of the paper's section
2.1 and the 2*CP mini-chunk rule of section 2.3); this module only compiles it
with gcc and marshals numpy arrays into it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hstu_oracle.c")
_SRC_BIAS = os.path.join(_HERE, "hstu_oracle_bias.c")
_LIB = os.path.join(_HERE, "libhstu_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with the host compiler; returns the library path."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_BIAS))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.run(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", tmp, _SRC, _SRC_BIAS, "-lm"],
            check=True,
        )
        os.replace(tmp, _LIB)
    return _LIB


_f64p = ctypes.POINTER(ctypes.c_double)
_i32p = ctypes.POINTER(ctypes.c_int32)
_i64p = ctypes.POINTER(ctypes.c_int64)


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.hstu_oracle_silu.restype = ctypes.c_double
        _lib.hstu_oracle_silu.argtypes = [ctypes.c_double]
        _lib.hstu_oracle_silu_grad.restype = ctypes.c_double
        _lib.hstu_oracle_silu_grad.argtypes = [ctypes.c_double]
        _lib.hstu_oracle_num_threads.restype = ctypes.c_int
        _lib.hstu_oracle_cp_local_rows.restype = ctypes.c_int64
        _lib.hstu_oracle_cp_local_map.restype = ctypes.c_int64
    return _lib


def _d(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: Optional[np.ndarray]):
    return a.ctypes.data_as(_f64p) if a is not None else None


def _off(off) -> np.ndarray:
    return np.ascontiguousarray(off, dtype=np.int32)


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError("%s failed with code %d" % (what, rc))


def num_threads() -> int:
    """Threads the oracle's parallel loops use."""
    return int(_load().hstu_oracle_num_threads())


def silu(x: float) -> float:
    return float(_load().hstu_oracle_silu(float(x)))


def silu_grad(x: float) -> float:
    return float(_load().hstu_oracle_silu_grad(float(x)))


def _dims(q, v, off):
    T, H, dqk = q.shape
    dv = v.shape[2]
    B = len(off) - 1
    assert off[0] == 0 and off[B] == T, "offsets must start at 0 and end at T"
    return T, H, dqk, dv, B


def fwd(q, k, v, off, max_len: int, alpha: float, causal: bool = True) -> np.ndarray:
    """O of the whole jagged batch; q,k: [T,H,d_qk], v: [T,H,d_v]; returns float64 [T,H,d_v]."""
    q, k, v, off = _d(q), _d(k), _d(v), _off(off)
    T, H, dqk, dv, B = _dims(q, v, off)
    o = np.zeros((T, H, dv), dtype=np.float64)
    rc = _load().hstu_oracle_fwd(
        ctypes.c_int32(B), ctypes.c_int32(H), ctypes.c_int32(dqk), ctypes.c_int32(dv),
        ctypes.c_int32(max_len), ctypes.c_double(alpha), ctypes.c_int32(int(causal)),
        off.ctypes.data_as(_i32p), _p(q), _p(k), _p(v), _p(o))
    _check(rc, "hstu_oracle_fwd")
    return o


def bwd(q, k, v, d_o, off, max_len: int, alpha: float, causal: bool = True
        ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(dQ, dK, dV) of the whole jagged batch, float64."""
    q, k, v, d_o, off = _d(q), _d(k), _d(v), _d(d_o), _off(off)
    T, H, dqk, dv, B = _dims(q, v, off)
    dq = np.zeros((T, H, dqk)); dk = np.zeros((T, H, dqk)); dvv = np.zeros((T, H, dv))
    rc = _load().hstu_oracle_bwd(
        ctypes.c_int32(B), ctypes.c_int32(H), ctypes.c_int32(dqk), ctypes.c_int32(dv),
        ctypes.c_int32(max_len), ctypes.c_double(alpha), ctypes.c_int32(int(causal)),
        off.ctypes.data_as(_i32p), _p(q), _p(k), _p(v), _p(d_o), _p(dq), _p(dk), _p(dvv))
    _check(rc, "hstu_oracle_bwd")
    return dq, dk, dvv


def rows(q, k, v, d_o, off, max_len: int, alpha: float, causal: bool, sel: Sequence[int],
         want_grads: bool = True):
    """Exact O, dQ, dK, dV at the global rows `sel` only: each [len(sel), H, d].

    With want_grads False (or d_o None) only O is computed and returned.
    """
    q, k, v, off = _d(q), _d(k), _d(v), _off(off)
    T, H, dqk, dv, B = _dims(q, v, off)
    sel = np.ascontiguousarray(sel, dtype=np.int64)
    n = len(sel)
    o = np.zeros((n, H, dv))
    grads = want_grads and d_o is not None
    if grads:
        d_o = _d(d_o)
        dq = np.zeros((n, H, dqk)); dk = np.zeros((n, H, dqk)); dvv = np.zeros((n, H, dv))
    else:
        d_o = dq = dk = dvv = None
    rc = _load().hstu_oracle_rows(
        ctypes.c_int32(B), ctypes.c_int32(H), ctypes.c_int32(dqk), ctypes.c_int32(dv),
        ctypes.c_int32(max_len), ctypes.c_double(alpha), ctypes.c_int32(int(causal)),
        off.ctypes.data_as(_i32p), _p(q), _p(k), _p(v), _p(d_o),
        ctypes.c_int32(n), sel.ctypes.data_as(_i64p), _p(o), _p(dq), _p(dk), _p(dvv))
    _check(rc, "hstu_oracle_rows")
    return (o, dq, dk, dvv) if grads else o


def cp_local_map(off, cp: int, rank: int) -> Tuple[np.ndarray, np.ndarray]:
    """(sequence index, in-sequence position) of every row of `rank`'s local layout.

    Local order: for each sequence in turn, mini-chunk `rank` then mini-chunk
    2*cp-1-rank (section 2.3's assignment).  rank < 0: all rows, global order.
    """
    off = _off(off)
    B = len(off) - 1
    lib = _load()
    n = lib.hstu_oracle_cp_local_rows(ctypes.c_int32(B), off.ctypes.data_as(_i32p),
                                      ctypes.c_int32(cp), ctypes.c_int32(rank))
    seq = np.zeros(n, dtype=np.int32); pos = np.zeros(n, dtype=np.int32)
    lib.hstu_oracle_cp_local_map(ctypes.c_int32(B), off.ctypes.data_as(_i32p),
                                 ctypes.c_int32(cp), ctypes.c_int32(rank),
                                 seq.ctypes.data_as(_i32p), pos.ctypes.data_as(_i32p))
    return seq, pos


def cp_global_rows(off, cp: int, rank: int) -> np.ndarray:
    """Global row index of every row of `rank`'s local layout (int64)."""
    off = _off(off)
    seq, pos = cp_local_map(off, cp, rank)
    return off[seq].astype(np.int64) + pos.astype(np.int64)


def cp_partial(q_local, k_part, v_part, d_o_local, off, max_len: int, alpha: float, causal: bool,
               cp: int, q_rank: int, kv_rank: int,
               sel_q: Optional[Sequence[int]] = None, sel_k: Optional[Sequence[int]] = None):
    """One rank's partial against kv_rank's keys (kv_rank < 0: all keys, global layout).

    Returns (o_local, dq_local, dk_part, dv_part); the gradients are None when
    d_o_local is None.  sel_q / sel_k restrict the computed rows (others stay 0).
    """
    q_local, k_part, v_part, off = _d(q_local), _d(k_part), _d(v_part), _off(off)
    nq, H, dqk = q_local.shape
    nk, _, dv = v_part.shape
    B = len(off) - 1
    o = np.zeros((nq, H, dv))
    if d_o_local is not None:
        d_o_local = _d(d_o_local)
        dq = np.zeros((nq, H, dqk)); dk = np.zeros((nk, H, dqk)); dvv = np.zeros((nk, H, dv))
    else:
        dq = dk = dvv = None
    sq = np.ascontiguousarray(sel_q, dtype=np.int64) if sel_q is not None else None
    sk = np.ascontiguousarray(sel_k, dtype=np.int64) if sel_k is not None else None
    rc = _load().hstu_oracle_cp_partial(
        ctypes.c_int32(B), ctypes.c_int32(H), ctypes.c_int32(dqk), ctypes.c_int32(dv),
        ctypes.c_int32(max_len), ctypes.c_double(alpha), ctypes.c_int32(int(causal)),
        off.ctypes.data_as(_i32p), ctypes.c_int32(cp), ctypes.c_int32(q_rank),
        ctypes.c_int32(kv_rank), _p(q_local), _p(k_part), _p(v_part), _p(d_o_local),
        _p(o), _p(dq), _p(dk), _p(dvv),
        ctypes.c_int64(len(sq) if sq is not None else -1),
        sq.ctypes.data_as(_i64p) if sq is not None else None,
        ctypes.c_int64(len(sk) if sk is not None else -1),
        sk.ctypes.data_as(_i64p) if sk is not None else None)
    _check(rc, "hstu_oracle_cp_partial")
    return o, dq, dk, dvv


def bias_bucket(ts_i: int, ts_j: int, nb: int, f: int) -> int:
    """Bucket of a timestamp difference (the reading in hstu_oracle_bias.c)."""
    lib = _load()
    lib.hstu_oracle_bias_bucket.restype = ctypes.c_int32
    return int(lib.hstu_oracle_bias_bucket(ctypes.c_int64(int(ts_i)), ctypes.c_int64(int(ts_j)),
                                           ctypes.c_int32(nb), ctypes.c_int32(f)))


def bias_attention(q, k, v, d_o, off, ts, w, f: int, max_len: int, alpha: float, causal: bool = True):
    """Attention with the timestamp bias: returns (o, dq, dk, dv, dw), the gradients None when
    d_o is None.  ts: int32 [T]; w: the bucket table [NB]; f: bits of groups per octave."""
    q, k, v, off = _d(q), _d(k), _d(v), _off(off)
    T, H, dqk, dv, B = _dims(q, v, off)
    ts = np.ascontiguousarray(ts, dtype=np.int32)
    w = _d(w)
    assert ts.shape == (T,)
    nb = len(w)
    o = np.zeros((T, H, dv), dtype=np.float64)
    back = d_o is not None
    d_o = _d(d_o) if back else None
    dq = np.zeros((T, H, dqk), dtype=np.float64) if back else None
    dk = np.zeros((T, H, dqk), dtype=np.float64) if back else None
    dvv = np.zeros((T, H, dv), dtype=np.float64) if back else None
    dw = np.zeros(nb, dtype=np.float64) if back else None
    rc = _load().hstu_oracle_bias(
        ctypes.c_int32(B), ctypes.c_int32(H), ctypes.c_int32(dqk), ctypes.c_int32(dv),
        ctypes.c_int32(max_len), ctypes.c_double(alpha), ctypes.c_int32(int(causal)),
        off.ctypes.data_as(_i32p), ts.ctypes.data_as(_i32p), ctypes.c_int32(nb), ctypes.c_int32(f),
        _p(w), _p(q), _p(k), _p(v), _p(d_o), _p(o), _p(dq), _p(dk), _p(dvv), _p(dw))
    _check(rc, "hstu_oracle_bias")
    return o, dq, dk, dvv, dw


def bias_rows(q, k, v, d_o, off, ts, w, f: int, max_len: int, alpha: float, causal: bool, sel):
    """Attention with the timestamp bias at the global rows `sel` only: (o, dq, dk, dv), each
    [len(sel), H, d] (the gradients None when d_o is None)."""
    q, k, v, off = _d(q), _d(k), _d(v), _off(off)
    T, H, dqk, dv, B = _dims(q, v, off)
    ts = np.ascontiguousarray(ts, dtype=np.int32)
    w = _d(w)
    sel = np.ascontiguousarray(sel, dtype=np.int64)
    n = len(sel)
    o = np.zeros((n, H, dv))
    back = d_o is not None
    d_o = _d(d_o) if back else None
    dq = np.zeros((n, H, dqk)) if back else None
    dk = np.zeros((n, H, dqk)) if back else None
    dvv = np.zeros((n, H, dv)) if back else None
    rc = _load().hstu_oracle_bias_rows(
        ctypes.c_int32(B), ctypes.c_int32(H), ctypes.c_int32(dqk), ctypes.c_int32(dv),
        ctypes.c_int32(max_len), ctypes.c_double(alpha), ctypes.c_int32(int(causal)),
        off.ctypes.data_as(_i32p), ts.ctypes.data_as(_i32p), ctypes.c_int32(len(w)), ctypes.c_int32(f),
        _p(w), _p(q), _p(k), _p(v), _p(d_o), ctypes.c_int32(n), sel.ctypes.data_as(_i64p),
        _p(o), _p(dq), _p(dk), _p(dvv))
    _check(rc, "hstu_oracle_bias_rows")
    return o, dq, dk, dvv

"""ctypes front end of the fp64 C oracle (``hg_oracle.c``) -- TEST INFRASTRUCTURE ONLY.

Argument marshalling only: numpy arrays in, numpy float64 arrays out.  q is ``[B, Hq, d]``;
K and V are ``[B, Hkv, Nmax, d]`` arrays (any strides over the first three axes, channel axis
contiguous) of dtype float16, float32, or uint16 holding bfloat16 bit patterns; ``seq_lens[b]`` tokens of sequence ``b`` are valid.
The routines and the passages of the paper they follow are described in ``hg_oracle.c``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hg_oracle.c")
_LIB = os.path.join(_HERE, "libhg_oracle.so")
_lock = threading.Lock()
_lib = None


class _Range(ctypes.Structure):
    _fields_ = [("seq", ctypes.c_int32), ("begin", ctypes.c_int32), ("end", ctypes.c_int32)]


class _Problem(ctypes.Structure):
    _fields_ = [
        ("q", ctypes.c_void_p),
        ("k", ctypes.c_void_p),
        ("v", ctypes.c_void_p),
        ("stride_b", ctypes.c_int64),
        ("stride_h", ctypes.c_int64),
        ("stride_t", ctypes.c_int64),
        ("seq_lens", ctypes.c_void_p),
        ("B", ctypes.c_int32),
        ("Hq", ctypes.c_int32),
        ("Hkv", ctypes.c_int32),
        ("d", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("scale", ctypes.c_double),
    ]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C11 + OpenMP).  Returns the library path."""
    with _lock:
        stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
        if force or stale:
            tmp = _LIB + ".tmp.%d" % os.getpid()
            subprocess.check_call(
                ["gcc", "-O2", "-std=c11", "-fopenmp", "-Wall", "-Wextra", "-shared", "-fPIC", _SRC, "-o", tmp, "-lm"]
            )
            os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        P = ctypes.POINTER(_Problem)
        dp = ctypes.c_void_p
        lib.hgo_attn_full.argtypes = [P, dp, dp, ctypes.c_int]
        lib.hgo_attn_partial.argtypes = [P, ctypes.POINTER(_Range), ctypes.c_int32, dp, dp, dp, ctypes.c_int]
        lib.hgo_attn_merge.argtypes = [dp, dp, dp, dp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, dp, dp]
        lib.hgo_attn_concat.argtypes = [P, ctypes.POINTER(_Range), ctypes.c_int32, dp, ctypes.c_int]
        lib.hgo_attn_logits.argtypes = [P, ctypes.POINTER(_Range), ctypes.c_int32, dp, ctypes.c_int]
        lib.hgo_attn_select.argtypes = [P, ctypes.POINTER(_Range), ctypes.c_int32, dp, dp, ctypes.c_int32, ctypes.c_int32,
                                        dp, dp, dp, dp]
        lib.hgo_attn_select.restype = ctypes.c_int
        lib.hgo_attn_gather.argtypes = [P, dp, ctypes.c_int32, dp, ctypes.c_int32, dp, dp, dp]
        lib.hgo_attn_gather.restype = ctypes.c_int
        for f in (lib.hgo_attn_full, lib.hgo_attn_partial, lib.hgo_attn_merge, lib.hgo_attn_concat, lib.hgo_attn_logits,
                  lib.hgo_max_threads):
            f.restype = ctypes.c_int
        _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().hgo_max_threads())


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError("oracle %s failed with code %d" % (what, rc))


def _problem(q, k, v, seq_lens, scale):
    q = np.ascontiguousarray(q)
    if q.dtype not in (np.float16, np.float32, np.uint16) or k.dtype != q.dtype or v.dtype != q.dtype:
        raise TypeError("q, k, v must share dtype float16, float32 or uint16 (bfloat16 bit patterns)")
    if q.ndim != 3 or k.ndim != 4 or v.ndim != 4 or k.shape != v.shape:
        raise ValueError("q must be [B,Hq,d]; k and v [B,Hkv,N,d] of equal shape")
    B, Hq, d = q.shape
    if k.shape[0] != B or k.shape[3] != d:
        raise ValueError("k/v do not match q")
    if k.strides != v.strides:
        raise ValueError("k and v must share strides")
    es = k.dtype.itemsize
    if B and k.shape[2] and k.strides[3] != es:
        raise ValueError("channel axis must be contiguous")
    seq = np.ascontiguousarray(seq_lens, dtype=np.int32)
    if seq.shape != (B,) or (B and (seq.min() < 0 or seq.max() > k.shape[2])):
        raise ValueError("seq_lens must be [B] with 0 <= N_b <= k.shape[2]")
    prob = _Problem(
        q.ctypes.data, k.ctypes.data, v.ctypes.data,
        k.strides[0] // es, k.strides[1] // es, k.strides[2] // es,
        seq.ctypes.data, B, Hq, k.shape[1], d, {np.dtype(np.float16): 0, np.dtype(np.float32): 1, np.dtype(np.uint16): 2}[q.dtype], float(scale),
    )
    return prob, (q, k, v, seq)  # second item keeps the buffers alive


def _ranges(ranges):
    arr = (_Range * max(len(ranges), 1))()
    for i, (s, b, e) in enumerate(ranges):
        arr[i] = _Range(int(s), int(b), int(e))
    return arr


def attn_full(q, k, v, seq_lens, scale, nthreads: int = 0):
    """Unsplit softmax attention.  Returns (out [B,Hq,d], lse [B,Hq]) in float64."""
    prob, keep = _problem(q, k, v, seq_lens, scale)
    out = np.zeros((prob.B, prob.Hq, prob.d), dtype=np.float64)
    lse = np.zeros((prob.B, prob.Hq), dtype=np.float64)
    _check(_load().hgo_attn_full(ctypes.byref(prob), out.ctypes.data, lse.ctypes.data, nthreads), "attn_full")
    del keep
    return out, lse


def attn_partial(q, k, v, seq_lens, scale, ranges, nthreads: int = 0):
    """Per-range statistics.  ranges: sequence of (seq, begin, end).
    Returns (m [R,Hq], l [R,Hq], o [R,Hq,d]) in float64."""
    prob, keep = _problem(q, k, v, seq_lens, scale)
    R = len(ranges)
    m = np.zeros((R, prob.Hq), dtype=np.float64)
    l = np.zeros((R, prob.Hq), dtype=np.float64)
    o = np.zeros((R, prob.Hq, prob.d), dtype=np.float64)
    arr = _ranges(ranges)
    _check(
        _load().hgo_attn_partial(ctypes.byref(prob), arr, R, m.ctypes.data, l.ctypes.data, o.ctypes.data, nthreads),
        "attn_partial",
    )
    del keep
    return m, l, o


def attn_merge(m, l, o, group_ptr):
    """Exact merge of triples.  m, l: [T,Hq]; o: [T,Hq,d]; group_ptr: CSR [n_groups+1].
    Returns (out [n_groups,Hq,d], lse [n_groups,Hq]) in float64."""
    m = np.ascontiguousarray(m, dtype=np.float64)
    l = np.ascontiguousarray(l, dtype=np.float64)
    o = np.ascontiguousarray(o, dtype=np.float64)
    gp = np.ascontiguousarray(group_ptr, dtype=np.int32)
    if o.ndim != 3 or m.shape != o.shape[:2] or l.shape != m.shape:
        raise ValueError("m, l must be [T,Hq] and o [T,Hq,d]")
    if gp.ndim != 1 or gp.size < 1 or gp[-1] > m.shape[0]:
        raise ValueError("group_ptr must be CSR offsets into the triples")
    n_groups = gp.size - 1
    _, Hq, d = o.shape
    out = np.zeros((n_groups, Hq, d), dtype=np.float64)
    lse = np.zeros((n_groups, Hq), dtype=np.float64)
    _check(
        _load().hgo_attn_merge(m.ctypes.data, l.ctypes.data, o.ctypes.data, gp.ctypes.data, n_groups, Hq, d,
                               out.ctypes.data, lse.ctypes.data),
        "attn_merge",
    )
    return out, lse


def attn_concat(q, k, v, seq_lens, scale, ranges, nthreads: int = 0):
    """Paper-literal route: logits of all ranges of a sequence concatenated in token order,
    one softmax, then P.V.  Returns out [B,Hq,d] in float64."""
    prob, keep = _problem(q, k, v, seq_lens, scale)
    out = np.zeros((prob.B, prob.Hq, prob.d), dtype=np.float64)
    arr = _ranges(ranges)
    _check(_load().hgo_attn_concat(ctypes.byref(prob), arr, len(ranges), out.ctypes.data, nthreads), "attn_concat")
    del keep
    return out


def attn_logits(q, k, v, seq_lens, scale, ranges, nthreads: int = 0):
    """Raw scaled logits of the listed ranges, concatenated in table order.
    Returns logits [Hq, ltok] in float64 (ltok = total length of the ranges)."""
    prob, keep = _problem(q, k, v, seq_lens, scale)
    ltok = sum(int(e) - int(b) for (_, b, e) in ranges)
    out = np.zeros((prob.Hq, ltok), dtype=np.float64)
    arr = _ranges(ranges)
    _check(_load().hgo_attn_logits(ctypes.byref(prob), arr, len(ranges), out.ctypes.data, nthreads), "attn_logits")
    del keep
    return out


def attn_select(q, k, v, seq_lens, scale, ranges, logits, group_ptr, top_k):
    """Post-QK^T selection on GIVEN fp32 logits [Hq, ltok]: per (group, head) keep the top_k
    logits (ties to the lower column) and fold them with their V rows into (m, l, O).
    Returns (sel int32 [G,Hq,top_k] token positions ascending, -1 padded; m, l [G,Hq]; o [G,Hq,d])."""
    prob, keep = _problem(q, k, v, seq_lens, scale)
    lg = np.ascontiguousarray(logits, dtype=np.float32)
    gp = np.ascontiguousarray(group_ptr, dtype=np.int32)
    ltok = sum(int(e) - int(b) for (_, b, e) in ranges)
    if lg.shape != (prob.Hq, ltok):
        raise ValueError("logits must be [Hq, ltok]")
    G = gp.size - 1
    sel = np.full((G, prob.Hq, top_k), -1, dtype=np.int32)
    m = np.zeros((G, prob.Hq), dtype=np.float64)
    l = np.zeros((G, prob.Hq), dtype=np.float64)
    o = np.zeros((G, prob.Hq, prob.d), dtype=np.float64)
    arr = _ranges(ranges)
    _check(_load().hgo_attn_select(ctypes.byref(prob), arr, len(ranges), lg.ctypes.data, gp.ctypes.data, G, int(top_k),
                                   sel.ctypes.data, m.ctypes.data, l.ctypes.data, o.ctypes.data), "attn_select")
    del keep
    return sel, m, l, o


def attn_gather(q, k, v, seq_lens, scale, group_seq, index):
    """Statistics over listed tokens: index int32 [G,Hq,max_k] positions of sequence group_seq[g]
    (negative = padding, duplicates count as often as listed).
    Returns (m [G,Hq], l [G,Hq], o [G,Hq,d]) in float64."""
    prob, keep = _problem(q, k, v, seq_lens, scale)
    gs = np.ascontiguousarray(group_seq, dtype=np.int32)
    idx = np.ascontiguousarray(index, dtype=np.int32)
    G = gs.size
    if idx.ndim != 3 or idx.shape[:2] != (G, prob.Hq) or idx.shape[2] < 1:
        raise ValueError("index must be [n_groups, Hq, max_k]")
    m = np.zeros((G, prob.Hq), dtype=np.float64)
    l = np.zeros((G, prob.Hq), dtype=np.float64)
    o = np.zeros((G, prob.Hq, prob.d), dtype=np.float64)
    _check(_load().hgo_attn_gather(ctypes.byref(prob), gs.ctypes.data, G, idx.ctypes.data, int(idx.shape[2]),
                                   m.ctypes.data, l.ctypes.data, o.ctypes.data), "attn_gather")
    del keep
    return m, l, o


def attn_topk(q, k, v, seq_lens, scale, ranges, group_ptr, top_k):
    """The Post-QK^T executor stage as one operation (Section 4.3.1; Section 4.6 step 1): the
    logits of the ranges with this query (attn_logits), rounded once to fp32 -- the precision in
    which the selection is decided -- then attn_select on them.  A composition of the two routines
    above, nothing else.  Returns (sel, m, l, o, logits_fp32)."""
    lg = attn_logits(q, k, v, seq_lens, scale, ranges).astype(np.float32)
    sel, m, l, o = attn_select(q, k, v, seq_lens, scale, ranges, lg, group_ptr, top_k)
    return sel, m, l, o, lg

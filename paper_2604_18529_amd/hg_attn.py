"""Thin Python binding of the C ABI in ``include/hg_attn.h``.

Argument marshalling only: every step of the attention path runs inside the HIP library.
PyTorch supplies device memory (tensors) and the stream; nothing here computes.
There is no fallback: if the library is missing and cannot be built, importing fails loudly.

Shapes (see the header for the full contract):
  q [B, Hq, d]; k, v [B, Hkv, N, d] (any strides over the first three axes, channel stride 1);
  seq_lens: host int32 [B]; ranges: sequence of (seq, begin, end) or a packed table from
  ``pack_ranges``; triples m, l [R, Hq] and o [R, Hq, d] in fp32.
"""
from __future__ import annotations

import ctypes
import math
import os
from typing import Optional, Sequence, Tuple

import numpy as np
import torch

from . import _build

HG_OK = 0
HG_F16, HG_F32, HG_BF16 = 0, 1, 2


class HgError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (what, hg_strerror(status), status))


class _Desc(ctypes.Structure):
    _fields_ = [
        ("q", ctypes.c_void_p),
        ("k", ctypes.c_void_p),
        ("v", ctypes.c_void_p),
        ("stride_b", ctypes.c_int64),
        ("stride_h", ctypes.c_int64),
        ("stride_t", ctypes.c_int64),
        ("seq_lens", ctypes.c_void_p),
        ("batch", ctypes.c_int32),
        ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("scale", ctypes.c_float),
        ("block_table", ctypes.c_void_p),
        ("block_tokens", ctypes.c_int32),
        ("max_blocks", ctypes.c_int32),
    ]


class HgSchedState(ctypes.Structure):
    """State of the feedback scheduler policy: k and strategy (0 = Post-QK^T, 1 = Pre-QK^T)."""

    _fields_ = [("k", ctypes.c_int32), ("strategy", ctypes.c_int32)]


class _Range(ctypes.Structure):
    _fields_ = [("seq", ctypes.c_int32), ("begin", ctypes.c_int32), ("end", ctypes.c_int32)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load ``libhg_attn.so``.  A binary that is missing, or that was built from other sources than
    the present ones (its build id is a hash of them), is rebuilt with hipcc first; if that is not
    possible the import fails rather than running a stale binary."""
    global _lib
    if _lib is not None:
        return _lib
    if _build.is_stale():
        _build.build_library()
    lib = ctypes.CDLL(_build.LIB_PATH)
    lib.hg_attn_build_id.restype = ctypes.c_char_p
    if lib.hg_attn_build_id().decode() != _build.source_id():
        raise RuntimeError("libhg_attn.so does not match the sources (build id %s, sources %s)"
                           % (lib.hg_attn_build_id().decode(), _build.source_id()))
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    D, R = ctypes.POINTER(_Desc), ctypes.POINTER(_Range)
    lib.hg_strerror.argtypes = [ctypes.c_int]
    lib.hg_strerror.restype = ctypes.c_char_p
    lib.hg_attn_partial_workspace_size.argtypes = [D, R, i32, ctypes.POINTER(sz)]
    lib.hg_attn_partial.argtypes = [D, R, i32, vp, vp, vp, vp, sz, vp]
    lib.hg_attn_partial_static.argtypes = [D, R, i32, vp, vp, vp, vp]
    lib.hg_attn_partial_merge_workspace_size.argtypes = [D, R, i32, vp, i32, ctypes.POINTER(sz)]
    lib.hg_attn_partial_merge.argtypes = [D, R, i32, vp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.hg_attn_merge_workspace_size.argtypes = [i32, ctypes.POINTER(sz)]
    lib.hg_attn_merge.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, sz, vp]
    lib.hg_attn_topk_workspace_size.argtypes = [D, R, i32, vp, i32, i32, ctypes.POINTER(sz)]
    lib.hg_attn_topk.argtypes = [D, R, i32, vp, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.hg_attn_gather_workspace_size.argtypes = [i32, ctypes.POINTER(sz)]
    lib.hg_attn_gather.argtypes = [ctypes.POINTER(_Desc), vp, i32, vp, i32, vp, vp, vp, vp, sz, vp]
    lib.hg_attn_merge2_workspace_size.argtypes = [i32, ctypes.POINTER(sz)]
    lib.hg_attn_merge2.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, sz, vp]
    lib.hg_attn_logits_workspace_size.argtypes = [D, R, i32, ctypes.POINTER(sz)]
    lib.hg_attn_logits.argtypes = [D, R, i32, vp, vp, sz, vp]
    lib.hg_attn_concat_workspace_size.argtypes = [D, R, i32, i32, ctypes.POINTER(sz)]
    lib.hg_attn_concat.argtypes = [D, R, i32, vp, vp, i32, vp, vp, vp, sz, vp]
    lib.hg_attn_select_workspace_size.argtypes = [D, R, i32, vp, i32, i32, ctypes.POINTER(sz)]
    lib.hg_attn_select.argtypes = [D, R, i32, vp, vp, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.hg_sched_init.argtypes = [ctypes.POINTER(HgSchedState), i32]
    lib.hg_sched_step.argtypes = [ctypes.POINTER(HgSchedState), ctypes.c_float, ctypes.c_float, ctypes.c_float, i32, i32, i32]
    lib.hg_attn_full_workspace_size.argtypes = [D, ctypes.POINTER(sz)]
    lib.hg_attn_full.argtypes = [D, vp, vp, vp, sz, vp]
    lib.hg_attn_plan.argtypes = [D, R, i32, ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_int64)]
    lib.hg_attn_set_span_tokens.argtypes = [i32]
    lib.hg_attn_set_topk_mode.argtypes = [i32]
    lib.hg_attn_profile_start.argtypes = [i32, i32]
    lib.hg_attn_calibration_copy.argtypes = [vp, vp, sz, vp]
    lib.hg_attn_calibration_stream.argtypes = [vp, sz, vp, i32, i32, i32, vp]
    lib.hg_attn_profile_stop.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i32)]
    lib.hg_attn_profile_times.argtypes = [ctypes.POINTER(ctypes.c_float), i32, ctypes.POINTER(i32)]
    for name in (
        "hg_attn_partial_workspace_size", "hg_attn_partial", "hg_attn_partial_static", "hg_attn_profile_times",
        "hg_attn_merge_workspace_size", "hg_attn_merge", "hg_attn_partial_merge_workspace_size", "hg_attn_partial_merge",
        "hg_attn_merge2_workspace_size", "hg_attn_merge2", "hg_attn_gather_workspace_size", "hg_attn_gather",
        "hg_attn_topk_workspace_size", "hg_attn_topk",
        "hg_attn_full_workspace_size", "hg_attn_full", "hg_attn_plan", "hg_attn_set_span_tokens", "hg_attn_set_topk_mode",
        "hg_attn_profile_start", "hg_attn_profile_stop", "hg_attn_calibration_copy", "hg_attn_calibration_stream",
        "hg_sched_init", "hg_sched_step", "hg_attn_logits_workspace_size", "hg_attn_logits", "hg_attn_select_workspace_size", "hg_attn_select", "hg_attn_concat_workspace_size", "hg_attn_concat",
    ):
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def hg_strerror(status: int) -> str:
    return load_library().hg_strerror(int(status)).decode()


def _check(status: int, what: str) -> None:
    if status != HG_OK:
        raise HgError(status, what)


def pack_ranges(ranges):
    """(seq, begin, end) triples -> packed hg_range array (reusable across calls)."""
    if isinstance(ranges, ctypes.Array):
        return ranges
    arr = (_Range * max(len(ranges), 1))()
    for i, (s, b, e) in enumerate(ranges):
        arr[i].seq, arr[i].begin, arr[i].end = int(s), int(b), int(e)
    arr.n = len(ranges)
    return arr


def _n_ranges(packed) -> int:
    return getattr(packed, "n", len(packed))


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream or None
    return int(stream) or None


def _note_stream(stream, *tensors) -> None:
    """Tensors the wrappers allocate (workspace, default outputs) come from torch's caching
    allocator on the CURRENT stream; the calls only enqueue work.  When the work goes to another
    torch stream, tell the allocator, so that a dropped tensor's block is not handed out again
    while that stream still uses it.  (A raw stream handle cannot be recorded: pass caller-owned
    buffers with it, as the C ABI requires anyway.)"""
    if isinstance(stream, torch.cuda.Stream) and stream != torch.cuda.current_stream(stream.device):
        for t in tensors:
            if t is not None:
                t.record_stream(stream)


def make_desc(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, seq_lens, scale: Optional[float] = None,
              block_table: Optional[torch.Tensor] = None):
    """Describe a problem.  Returns (desc, keepalive); keepalive must outlive the calls using desc.

    Contiguous cache: k, v are [B, Hkv, N, d].  Paged cache (``block_table`` int32 [B, max_blocks]
    on the device): k, v are the physical pools [n_blocks, Hkv, block_tokens, d]."""
    if q.dtype not in (torch.float16, torch.float32, torch.bfloat16) or k.dtype != q.dtype or v.dtype != q.dtype:
        raise TypeError("q, k, v must share dtype float16, bfloat16 or float32")
    if q.dim() != 3 or k.dim() != 4 or v.dim() != 4 or k.shape != v.shape:
        raise ValueError("q must be [B,Hq,d]; k and v [B,Hkv,N,d] (or [blocks,Hkv,block_tokens,d]) of equal shape")
    if not q.is_contiguous():
        raise ValueError("q must be contiguous")
    B, Hq, d = q.shape
    if k.shape[3] != d or (block_table is None and k.shape[0] != B):
        raise ValueError("k/v do not match q")
    if k.stride() != v.stride() or (k.numel() and k.stride(3) != 1):
        raise ValueError("k and v must share strides and have a contiguous channel axis")
    if not (q.device == k.device == v.device):
        raise ValueError("q, k, v must live on one device")
    seq = np.ascontiguousarray(seq_lens, dtype=np.int32)
    if seq.shape != (B,):
        raise ValueError("seq_lens must be [B]")
    bt_ptr, block_tokens, max_blocks = None, 0, 0
    if block_table is None:
        if B and int(seq.max()) > k.shape[2]:
            raise ValueError("seq_lens exceeds the cache length")
    else:
        if block_table.dtype != torch.int32 or block_table.dim() != 2 or block_table.shape[0] != B or \
                not block_table.is_contiguous() or block_table.device != q.device:
            raise ValueError("block_table must be a contiguous int32 [B, max_blocks] tensor on q's device")
        bt_ptr, block_tokens, max_blocks = block_table.data_ptr(), int(k.shape[2]), int(block_table.shape[1])
    desc = _Desc(
        q.data_ptr(), k.data_ptr(), v.data_ptr(), k.stride(0), k.stride(1), k.stride(2), seq.ctypes.data,
        B, Hq, k.shape[1], d, {torch.float16: HG_F16, torch.float32: HG_F32, torch.bfloat16: HG_BF16}[q.dtype],
        float(scale if scale is not None else 1.0 / math.sqrt(d)), bt_ptr, block_tokens, max_blocks,
    )
    return desc, (q, k, v, seq, block_table)


def _workspace(nbytes: int, device, workspace: Optional[torch.Tensor]) -> Tuple[Optional[torch.Tensor], int]:
    if workspace is not None:
        return workspace, workspace.numel() * workspace.element_size()
    if nbytes == 0:
        return None, 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    return ws, nbytes


def hg_attn_plan(q, k, v, seq_lens, ranges, scale=None) -> Tuple[int, int]:
    """(span_tokens, n_workgroups) the library would use; host only."""
    lib = load_library()
    desc, keep = make_desc(q, k, v, seq_lens, scale)
    packed = pack_ranges(ranges)
    span = ctypes.c_int32()
    n = ctypes.c_int64()
    _check(lib.hg_attn_plan(ctypes.byref(desc), packed, _n_ranges(packed), ctypes.byref(span), ctypes.byref(n)), "hg_attn_plan")
    del keep
    return span.value, n.value


def hg_attn_set_span_tokens(span_tokens: int) -> None:
    _check(load_library().hg_attn_set_span_tokens(int(span_tokens)), "hg_attn_set_span_tokens")


def hg_attn_set_topk_mode(mode: int) -> None:
    """0: the library chooses; 1: filtering scan wherever it exists; 2: always logits -> select."""
    _check(load_library().hg_attn_set_topk_mode(int(mode)), "hg_attn_set_topk_mode")


def hg_attn_profile_start(max_calls: int, repeat: int = 1) -> None:
    _check(load_library().hg_attn_profile_start(int(max_calls), int(repeat)), "hg_attn_profile_start")


def hg_attn_profile_stop() -> Tuple[float, int]:
    """(summed milliseconds of the streaming kernel, launches timed)."""
    ms, n = ctypes.c_float(), ctypes.c_int32()
    _check(load_library().hg_attn_profile_stop(ctypes.byref(ms), ctypes.byref(n)), "hg_attn_profile_stop")
    return ms.value, n.value


def hg_attn_profile_times(capacity: int):
    """Milliseconds of one launch of the streaming kernel for each timed call so far (waits for them)."""
    buf = (ctypes.c_float * max(int(capacity), 1))()
    n = ctypes.c_int32()
    _check(load_library().hg_attn_profile_times(buf, int(capacity), ctypes.byref(n)), "hg_attn_profile_times")
    return [buf[i] for i in range(min(n.value, int(capacity)))]


def hg_attn_build_id() -> str:
    return load_library().hg_attn_build_id().decode()


def hg_attn_calibration_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    """Plain device copy of known traffic (profiler yardstick)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes or not (dst.is_contiguous() and src.is_contiguous()):
        raise ValueError("dst and src must be contiguous and of equal size")
    with torch.cuda.device(src.device):
        st = load_library().hg_attn_calibration_copy(dst.data_ptr(), src.data_ptr(), nbytes, _stream_handle(stream))
    _check(st, "hg_attn_calibration_copy")


def hg_attn_calibration_stream(src: torch.Tensor, read_bytes: int, dst: Optional[torch.Tensor] = None, write_vectors: int = 0,
                               burst_iterations: int = 1, streaming_stores: bool = False, stream=None) -> None:
    """Plain read stream of `read_bytes` bytes of src, optionally next to writes into dst (see the debug header)."""
    with torch.cuda.device(src.device):
        st = load_library().hg_attn_calibration_stream(src.data_ptr(), int(read_bytes), _ptr(dst), int(write_vectors),
                                                       int(burst_iterations), int(bool(streaming_stores)), _stream_handle(stream))
    _check(st, "hg_attn_calibration_stream")


def hg_attn_partial_workspace_size(desc, packed) -> int:
    sz = ctypes.c_size_t()
    _check(load_library().hg_attn_partial_workspace_size(ctypes.byref(desc), packed, _n_ranges(packed), ctypes.byref(sz)),
           "hg_attn_partial_workspace_size")
    return sz.value


def hg_attn_partial(q, k, v, seq_lens, ranges, scale=None, *, m=None, l=None, o=None, workspace=None, stream=None,
                    desc=None, block_table=None):
    """Per-range statistics.  Returns (m [R,Hq], l [R,Hq], o [R,Hq,d]) fp32 device tensors."""
    lib = load_library()
    if desc is None:
        desc, keep = make_desc(q, k, v, seq_lens, scale, block_table)
    else:
        keep = None
    packed = pack_ranges(ranges)
    R = _n_ranges(packed)
    dev = q.device
    Hq, d = q.shape[1], q.shape[2]
    if m is None:
        m = torch.empty((R, Hq), dtype=torch.float32, device=dev)
    if l is None:
        l = torch.empty((R, Hq), dtype=torch.float32, device=dev)
    if o is None:
        o = torch.empty((R, Hq, d), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace, ws_bytes = _workspace(hg_attn_partial_workspace_size(desc, packed), dev, None)
    else:
        ws_bytes = workspace.numel() * workspace.element_size()
    with torch.cuda.device(dev):
        st = lib.hg_attn_partial(ctypes.byref(desc), packed, R, _ptr(m), _ptr(l), _ptr(o), _ptr(workspace), ws_bytes,
                                 _stream_handle(stream))
    _check(st, "hg_attn_partial")
    _note_stream(stream, m, l, o, workspace)
    del keep
    return m, l, o


def hg_attn_partial_static(q, k, v, seq_lens, ranges, scale=None, *, m=None, l=None, o=None, stream=None, desc=None,
                           block_table=None):
    """hg_attn_partial with the library's static scratch buffer instead of a workspace (the C
    call allocates nothing; problems that need more scratch than it holds are refused)."""
    lib = load_library()
    if desc is None:
        desc, keep = make_desc(q, k, v, seq_lens, scale, block_table)
    else:
        keep = None
    packed = pack_ranges(ranges)
    R = _n_ranges(packed)
    dev = q.device
    Hq, d = q.shape[1], q.shape[2]
    if m is None:
        m = torch.empty((R, Hq), dtype=torch.float32, device=dev)
    if l is None:
        l = torch.empty((R, Hq), dtype=torch.float32, device=dev)
    if o is None:
        o = torch.empty((R, Hq, d), dtype=torch.float32, device=dev)
    with torch.cuda.device(dev):
        st = lib.hg_attn_partial_static(ctypes.byref(desc), packed, R, _ptr(m), _ptr(l), _ptr(o), _stream_handle(stream))
    _check(st, "hg_attn_partial_static")
    _note_stream(stream, m, l, o)
    del keep
    return m, l, o


def hg_attn_partial_merge_workspace_size(desc, packed_ranges, group_ptr) -> int:
    gp = np.ascontiguousarray(group_ptr, dtype=np.int32)
    sz = ctypes.c_size_t()
    _check(load_library().hg_attn_partial_merge_workspace_size(ctypes.byref(desc), packed_ranges, _n_ranges(packed_ranges),
                                                               gp.ctypes.data, gp.size - 1, ctypes.byref(sz)),
           "hg_attn_partial_merge_workspace_size")
    return sz.value


def hg_attn_partial_merge(q, k, v, seq_lens, ranges, group_ptr, scale=None, *, m=None, l=None, o=None, out=None, lse=None,
                          want_lse=True, workspace=None, stream=None, desc=None, block_table=None):
    """hg_attn_partial and hg_attn_merge in one call (one kernel launch on small inputs).
    Returns (m, l, o, out, lse)."""
    lib = load_library()
    if desc is None:
        desc, keep = make_desc(q, k, v, seq_lens, scale, block_table)
    else:
        keep = None
    packed = pack_ranges(ranges)
    R = _n_ranges(packed)
    gp = np.ascontiguousarray(group_ptr, dtype=np.int32)
    if gp.ndim != 1 or gp.size < 1:
        raise ValueError("group_ptr must be CSR offsets [n_groups+1]")
    n_groups = gp.size - 1
    dev = q.device
    Hq, d = q.shape[1], q.shape[2]
    if m is None:
        m = torch.empty((R, Hq), dtype=torch.float32, device=dev)
    if l is None:
        l = torch.empty((R, Hq), dtype=torch.float32, device=dev)
    if o is None:
        o = torch.empty((R, Hq, d), dtype=torch.float32, device=dev)
    if out is None:
        out = torch.empty((n_groups, Hq, d), dtype=torch.float32, device=dev)
    if lse is None and want_lse:
        lse = torch.empty((n_groups, Hq), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace, ws_bytes = _workspace(hg_attn_partial_merge_workspace_size(desc, packed, gp), dev, None)
    else:
        ws_bytes = workspace.numel() * workspace.element_size()
    with torch.cuda.device(dev):
        st = lib.hg_attn_partial_merge(ctypes.byref(desc), packed, R, gp.ctypes.data, n_groups, _ptr(m), _ptr(l), _ptr(o),
                                       _ptr(out), _ptr(lse), _ptr(workspace), ws_bytes, _stream_handle(stream))
    _check(st, "hg_attn_partial_merge")
    _note_stream(stream, m, l, o, out, lse, workspace)
    del keep
    return m, l, o, out, lse


def hg_attn_merge(m, l, o, group_ptr, *, out=None, lse=None, want_lse=True, workspace=None, stream=None):
    """Exact merge of triples per CSR group.  Returns (out [n_groups,Hq,d], lse [n_groups,Hq] or None)."""
    lib = load_library()
    gp = np.ascontiguousarray(group_ptr, dtype=np.int32)
    if gp.ndim != 1 or gp.size < 1:
        raise ValueError("group_ptr must be CSR offsets [n_groups+1]")
    if o.dim() != 3 or tuple(m.shape) != tuple(o.shape[:2]) or m.shape != l.shape:
        raise ValueError("m, l must be [T,Hq] and o [T,Hq,d]")
    for t in (m, l, o):
        if t.dtype != torch.float32 or not t.is_contiguous():
            raise ValueError("triples must be contiguous fp32")
    if gp[-1] > m.shape[0]:
        raise ValueError("group_ptr runs past the triples")
    n_groups = gp.size - 1
    _, Hq, d = o.shape
    dev = o.device
    if out is None:
        out = torch.empty((n_groups, Hq, d), dtype=torch.float32, device=dev)
    if lse is None and want_lse:
        lse = torch.empty((n_groups, Hq), dtype=torch.float32, device=dev)
    if workspace is None:
        sz = ctypes.c_size_t()
        _check(lib.hg_attn_merge_workspace_size(n_groups, ctypes.byref(sz)), "hg_attn_merge_workspace_size")
        workspace, ws_bytes = _workspace(sz.value, dev, None)
    else:
        ws_bytes = workspace.numel() * workspace.element_size()
    with torch.cuda.device(dev):
        st = lib.hg_attn_merge(_ptr(m), _ptr(l), _ptr(o), gp.ctypes.data, n_groups, Hq, d, _ptr(out), _ptr(lse),
                               _ptr(workspace), ws_bytes, _stream_handle(stream))
    _check(st, "hg_attn_merge")
    _note_stream(stream, out, lse, workspace)
    return out, lse


def _check_triples(m, l, o, gp, what):
    if o.dim() != 3 or tuple(m.shape) != tuple(o.shape[:2]) or m.shape != l.shape:
        raise ValueError("%s: m, l must be [T,Hq] and o [T,Hq,d]" % what)
    for t in (m, l, o):
        if t.dtype != torch.float32 or not t.is_contiguous():
            raise ValueError("%s: triples must be contiguous fp32" % what)
    if gp.ndim != 1 or gp.size < 1:
        raise ValueError("%s: group_ptr must be CSR offsets [n_groups+1]" % what)
    if gp[-1] > m.shape[0]:
        raise ValueError("%s: group_ptr runs past the triples" % what)


def hg_attn_merge2(m_a, l_a, o_a, group_ptr_a, m_b, l_b, o_b, group_ptr_b, *, out=None, lse=None, want_lse=True,
                   workspace=None, stream=None):
    """Exact merge of the triples of two producers (each with its own arrays and CSR) per group.
    Returns (out [n_groups,Hq,d], lse [n_groups,Hq] or None)."""
    lib = load_library()
    gpa = np.ascontiguousarray(group_ptr_a, dtype=np.int32)
    gpb = np.ascontiguousarray(group_ptr_b, dtype=np.int32)
    _check_triples(m_a, l_a, o_a, gpa, "set A")
    _check_triples(m_b, l_b, o_b, gpb, "set B")
    if gpa.size != gpb.size or o_a.shape[1:] != o_b.shape[1:]:
        raise ValueError("the two sets must agree in groups, heads and head_dim")
    n_groups = gpa.size - 1
    _, Hq, d = o_a.shape
    dev = o_a.device
    if out is None:
        out = torch.empty((n_groups, Hq, d), dtype=torch.float32, device=dev)
    if lse is None and want_lse:
        lse = torch.empty((n_groups, Hq), dtype=torch.float32, device=dev)
    if workspace is None:
        sz = ctypes.c_size_t()
        _check(lib.hg_attn_merge2_workspace_size(n_groups, ctypes.byref(sz)), "hg_attn_merge2_workspace_size")
        workspace, ws_bytes = _workspace(sz.value, dev, None)
    else:
        ws_bytes = workspace.numel() * workspace.element_size()
    with torch.cuda.device(dev):
        st = lib.hg_attn_merge2(_ptr(m_a), _ptr(l_a), _ptr(o_a), gpa.ctypes.data, _ptr(m_b), _ptr(l_b), _ptr(o_b),
                                gpb.ctypes.data, n_groups, Hq, d, _ptr(out), _ptr(lse), _ptr(workspace), ws_bytes,
                                _stream_handle(stream))
    _check(st, "hg_attn_merge2")
    _note_stream(stream, out, lse, workspace)
    return out, lse


def hg_attn_full_workspace_size(desc) -> int:
    sz = ctypes.c_size_t()
    _check(load_library().hg_attn_full_workspace_size(ctypes.byref(desc), ctypes.byref(sz)), "hg_attn_full_workspace_size")
    return sz.value


def hg_attn_full(q, k, v, seq_lens, scale=None, *, out=None, lse=None, want_lse=True, workspace=None, stream=None,
                 desc=None, block_table=None):
    """Unsplit attention over the whole cache.  Returns (out [B,Hq,d], lse [B,Hq] or None)."""
    lib = load_library()
    if desc is None:
        desc, keep = make_desc(q, k, v, seq_lens, scale, block_table)
    else:
        keep = None
    dev = q.device
    B, Hq, d = q.shape
    if out is None:
        out = torch.empty((B, Hq, d), dtype=torch.float32, device=dev)
    if lse is None and want_lse:
        lse = torch.empty((B, Hq), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace, ws_bytes = _workspace(hg_attn_full_workspace_size(desc), dev, None)
    else:
        ws_bytes = workspace.numel() * workspace.element_size()
    with torch.cuda.device(dev):
        st = lib.hg_attn_full(ctypes.byref(desc), _ptr(out), _ptr(lse), _ptr(workspace), ws_bytes, _stream_handle(stream))
    _check(st, "hg_attn_full")
    _note_stream(stream, out, lse, workspace)
    del keep
    return out, lse


def hg_attn_logits(q, k, v, seq_lens, ranges, scale=None, *, logits=None, workspace=None, stream=None, desc=None,
                   block_table=None):
    """Raw scaled logits of the listed ranges, concatenated in table order: fp32 [Hq, ltok]."""
    lib = load_library()
    if desc is None:
        desc, keep = make_desc(q, k, v, seq_lens, scale, block_table)
    else:
        keep = None
    packed = pack_ranges(ranges)
    R = _n_ranges(packed)
    ltok = sum(packed[i].end - packed[i].begin for i in range(R))
    dev = q.device
    if logits is None:
        logits = torch.empty((q.shape[1], ltok), dtype=torch.float32, device=dev)
    elif tuple(logits.shape) != (q.shape[1], ltok) or logits.dtype != torch.float32 or not logits.is_contiguous():
        raise ValueError("logits must be contiguous fp32 [Hq, ltok]")
    if workspace is None:
        sz = ctypes.c_size_t()
        _check(lib.hg_attn_logits_workspace_size(ctypes.byref(desc), packed, R, ctypes.byref(sz)), "hg_attn_logits_workspace_size")
        workspace, ws_bytes = _workspace(sz.value, dev, None)
    else:
        ws_bytes = workspace.numel() * workspace.element_size()
    with torch.cuda.device(dev):
        st = lib.hg_attn_logits(ctypes.byref(desc), packed, R, _ptr(logits), _ptr(workspace), ws_bytes, _stream_handle(stream))
    _check(st, "hg_attn_logits")
    _note_stream(stream, logits, workspace)
    del keep
    return logits


def hg_attn_concat_workspace_size(desc, packed, n_groups) -> int:
    sz = ctypes.c_size_t()
    _check(load_library().hg_attn_concat_workspace_size(ctypes.byref(desc), packed, _n_ranges(packed), int(n_groups),
                                                        ctypes.byref(sz)), "hg_attn_concat_workspace_size")
    return sz.value


def hg_attn_concat(q, k, v, seq_lens, ranges, logits, group_ptr, scale=None, *, out=None, lse=None, want_lse=True,
                   workspace=None, stream=None, desc=None, block_table=None):
    """One softmax over the concatenated logits of each group, then P.V (the paper-literal merge).
    Returns (out [n_groups,Hq,d], lse [n_groups,Hq] or None)."""
    lib = load_library()
    if desc is None:
        desc, keep = make_desc(q, k, v, seq_lens, scale, block_table)
    else:
        keep = None
    packed = pack_ranges(ranges)
    R = _n_ranges(packed)
    gp = np.ascontiguousarray(group_ptr, dtype=np.int32)
    if gp.ndim != 1 or gp.size < 1:
        raise ValueError("group_ptr must be CSR offsets [n_groups+1]")
    n_groups = gp.size - 1
    if logits.dtype != torch.float32 or not logits.is_contiguous() or logits.dim() != 2 or logits.shape[0] != q.shape[1]:
        raise ValueError("logits must be contiguous fp32 [Hq, ltok]")
    if logits.shape[1] != sum(packed[i].end - packed[i].begin for i in range(R)):
        raise ValueError("logits do not match the range table")
    dev = q.device
    Hq, d = q.shape[1], q.shape[2]
    if out is None:
        out = torch.empty((n_groups, Hq, d), dtype=torch.float32, device=dev)
    if lse is None and want_lse:
        lse = torch.empty((n_groups, Hq), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace, ws_bytes = _workspace(hg_attn_concat_workspace_size(desc, packed, n_groups), dev, None)
    else:
        ws_bytes = workspace.numel() * workspace.element_size()
    with torch.cuda.device(dev):
        st = lib.hg_attn_concat(ctypes.byref(desc), packed, R, _ptr(logits), gp.ctypes.data, n_groups, _ptr(out), _ptr(lse),
                                _ptr(workspace), ws_bytes, _stream_handle(stream))
    _check(st, "hg_attn_concat")
    _note_stream(stream, out, lse, workspace)
    del keep
    return out, lse


def hg_attn_select(q, k, v, seq_lens, ranges, logits, group_ptr, top_k, scale=None, *, want_sel=True, workspace=None,
                   stream=None, desc=None, block_table=None):
    """Post-QK^T selection: per (group, head) keep the top_k logits and fold them with their V rows.
    Returns (sel int32 [G,Hq,top_k] or None, m [G,Hq], l [G,Hq], o [G,Hq,d])."""
    lib = load_library()
    if desc is None:
        desc, keep = make_desc(q, k, v, seq_lens, scale, block_table)
    else:
        keep = None
    packed = pack_ranges(ranges)
    R = _n_ranges(packed)
    gp = np.ascontiguousarray(group_ptr, dtype=np.int32)
    if gp.ndim != 1 or gp.size < 1:
        raise ValueError("group_ptr must be CSR offsets [n_groups+1]")
    G = gp.size - 1
    if logits.dtype != torch.float32 or not logits.is_contiguous() or logits.dim() != 2 or logits.shape[0] != q.shape[1]:
        raise ValueError("logits must be contiguous fp32 [Hq, ltok]")
    if logits.shape[1] != sum(packed[i].end - packed[i].begin for i in range(R)):
        raise ValueError("logits do not match the range table")
    dev = q.device
    Hq, d = q.shape[1], q.shape[2]
    sel = torch.empty((G, Hq, int(top_k)), dtype=torch.int32, device=dev) if want_sel else None
    m = torch.empty((G, Hq), dtype=torch.float32, device=dev)
    l = torch.empty((G, Hq), dtype=torch.float32, device=dev)
    o = torch.empty((G, Hq, d), dtype=torch.float32, device=dev)
    if workspace is None:
        sz = ctypes.c_size_t()
        _check(lib.hg_attn_select_workspace_size(ctypes.byref(desc), packed, R, gp.ctypes.data, G, int(top_k), ctypes.byref(sz)),
               "hg_attn_select_workspace_size")
        workspace, ws_bytes = _workspace(sz.value, dev, None)
    else:
        ws_bytes = workspace.numel() * workspace.element_size()
    with torch.cuda.device(dev):
        st = lib.hg_attn_select(ctypes.byref(desc), packed, R, _ptr(logits), gp.ctypes.data, G, int(top_k), _ptr(sel),
                                _ptr(m), _ptr(l), _ptr(o), _ptr(workspace), ws_bytes, _stream_handle(stream))
    _check(st, "hg_attn_select")
    _note_stream(stream, sel, m, l, o, workspace)
    del keep
    return sel, m, l, o


def hg_attn_topk_workspace_size(desc, packed, group_ptr, top_k) -> int:
    gp = np.ascontiguousarray(group_ptr, dtype=np.int32)
    sz = ctypes.c_size_t()
    _check(load_library().hg_attn_topk_workspace_size(ctypes.byref(desc), packed, _n_ranges(packed), gp.ctypes.data, gp.size - 1,
                                                      int(top_k), ctypes.byref(sz)), "hg_attn_topk_workspace_size")
    return sz.value


def hg_attn_topk(q, k, v, seq_lens, ranges, group_ptr, top_k, scale=None, *, want_sel=True, workspace=None, stream=None,
                 desc=None, block_table=None):
    """Post-QK^T executor stage in one call: logits of the ranges, top_k per (group, head), kept
    tokens folded with their V rows.  Returns (sel int32 [G,Hq,top_k] or None, m, l [G,Hq], o [G,Hq,d])."""
    lib = load_library()
    if desc is None:
        desc, keep = make_desc(q, k, v, seq_lens, scale, block_table)
    else:
        keep = None
    packed = pack_ranges(ranges)
    R = _n_ranges(packed)
    gp = np.ascontiguousarray(group_ptr, dtype=np.int32)
    if gp.ndim != 1 or gp.size < 1:
        raise ValueError("group_ptr must be CSR offsets [n_groups+1]")
    G = gp.size - 1
    dev = q.device
    Hq, d = q.shape[1], q.shape[2]
    sel = torch.empty((G, Hq, int(top_k)), dtype=torch.int32, device=dev) if want_sel else None
    m = torch.empty((G, Hq), dtype=torch.float32, device=dev)
    l = torch.empty((G, Hq), dtype=torch.float32, device=dev)
    o = torch.empty((G, Hq, d), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace, ws_bytes = _workspace(hg_attn_topk_workspace_size(desc, packed, gp, top_k), dev, None)
    else:
        ws_bytes = workspace.numel() * workspace.element_size()
    with torch.cuda.device(dev):
        st = lib.hg_attn_topk(ctypes.byref(desc), packed, R, gp.ctypes.data, G, int(top_k), _ptr(sel), _ptr(m), _ptr(l),
                              _ptr(o), _ptr(workspace), ws_bytes, _stream_handle(stream))
    _check(st, "hg_attn_topk")
    _note_stream(stream, sel, m, l, o, workspace)
    del keep
    return sel, m, l, o


def hg_attn_gather(q, k, v, seq_lens, group_seq, index, scale=None, *, m=None, l=None, o=None, workspace=None,
                   stream=None, desc=None, block_table=None):
    """Statistics over listed tokens: index int32 [G,Hq,max_k] (negative = padding) of sequence
    group_seq[g].  Returns (m [G,Hq], l [G,Hq], o [G,Hq,d])."""
    lib = load_library()
    if desc is None:
        desc, keep = make_desc(q, k, v, seq_lens, scale, block_table)
    else:
        keep = None
    gs = np.ascontiguousarray(group_seq, dtype=np.int32)
    G = gs.size
    Hq, d = q.shape[1], q.shape[2]
    if index.dtype != torch.int32 or not index.is_contiguous() or index.dim() != 3 or tuple(index.shape[:2]) != (G, Hq):
        raise ValueError("index must be contiguous int32 [n_groups, Hq, max_k]")
    dev = q.device
    if m is None:
        m = torch.empty((G, Hq), dtype=torch.float32, device=dev)
    if l is None:
        l = torch.empty((G, Hq), dtype=torch.float32, device=dev)
    if o is None:
        o = torch.empty((G, Hq, d), dtype=torch.float32, device=dev)
    if workspace is None:
        sz = ctypes.c_size_t()
        _check(lib.hg_attn_gather_workspace_size(G, ctypes.byref(sz)), "hg_attn_gather_workspace_size")
        workspace, ws_bytes = _workspace(sz.value, dev, None)
    else:
        ws_bytes = workspace.numel() * workspace.element_size()
    with torch.cuda.device(dev):
        st = lib.hg_attn_gather(ctypes.byref(desc), gs.ctypes.data, G, _ptr(index), int(index.shape[2]), _ptr(m), _ptr(l),
                                _ptr(o), _ptr(workspace), ws_bytes, _stream_handle(stream))
    _check(st, "hg_attn_gather")
    _note_stream(stream, m, l, o, workspace)
    del keep
    return m, l, o


def hg_sched_init(k_min: int) -> HgSchedState:
    st = HgSchedState()
    _check(load_library().hg_sched_init(ctypes.byref(st), int(k_min)), "hg_sched_init")
    return st


def hg_sched_step(state: HgSchedState, t_gpu: float, t_cpu: float, t_tx: float, k_min: int, k_max: int, k_step: int):
    """One tick of the feedback scheduler policy; updates and returns (k, strategy)."""
    _check(load_library().hg_sched_step(ctypes.byref(state), float(t_gpu), float(t_cpu), float(t_tx), int(k_min), int(k_max),
                                        int(k_step)), "hg_sched_step")
    return state.k, state.strategy

"""Host-side checks of the C ABI (no GPU, no device work).

The library must load, export every function the header declares, reject malformed arguments
with the documented status before anything is enqueued, and plan tiles that cover every range
exactly once.  Pointers handed over here are fake non-NULL addresses: only calls that fail validation
(or that are host-only by contract) are made, so nothing is ever dereferenced on a device.
"""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2604_18529_amd import _build
from paper_2604_18529_amd import hg_attn as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", "hg_attn.h"), os.path.join(ROOT, "include", "hg_attn_debug.h")]

FAKE = 0x10000  # 16- and 256-byte aligned, never dereferenced


@pytest.fixture(scope="module")
def lib():
    if _build.is_stale():
        _build.build_library()
    return B.load_library()


def _desc(seq_lens, batch=None, hq=4, hkv=2, d=128, dtype=0, stride_t=None, q=FAKE, k=FAKE, v=FAKE, scale=0.1):
    seq = np.ascontiguousarray(seq_lens, dtype=np.int32)
    batch = len(seq) if batch is None else batch
    stride_t = d if stride_t is None else stride_t
    nmax = max(int(seq.max()), 1) if len(seq) else 1
    desc = B._Desc(q, k, v, hkv * nmax * stride_t, nmax * stride_t, stride_t, seq.ctypes.data, batch, hq, hkv, d, dtype, scale,
                   None, 0, 0)
    desc._keep = seq
    return desc


def _declared(header):
    text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
    return set(re.findall(r"\b(hg_[a-z_0-9]+)\s*\(", text))


def test_exports_every_declared_function(lib):
    method, aids = _declared(HEADERS[0]), _declared(HEADERS[1])
    assert {"hg_attn_partial", "hg_attn_merge", "hg_attn_full", "hg_strerror", "hg_attn_partial_static",
            "hg_attn_build_id"} <= method
    # process-wide knobs and blocking measurement aids live in the debug header only
    assert {"hg_attn_set_span_tokens", "hg_attn_set_topk_mode", "hg_attn_profile_start", "hg_attn_profile_times",
            "hg_attn_profile_stop", "hg_attn_calibration_copy", "hg_attn_calibration_stream"} <= aids
    assert not (method & aids)
    for n in sorted(method | aids):
        assert hasattr(lib, n), "library does not export %s" % n


def test_binary_matches_the_sources(lib):
    """The binary carries a hash of the sources it was built from; the loader compares it."""
    assert B.hg_attn_build_id() == _build.source_id() == _build.binary_id()
    assert not _build.is_stale()


def test_static_scratch_entry_point_validates_like_partial(lib):
    """hg_attn_partial_static: the same validation as hg_attn_partial, and problems whose segment
    records do not fit the static buffer are refused before anything is enqueued."""
    good = B.pack_ranges([(0, 0, 10)])

    def call(desc, packed=good, n=1, m=FAKE, l=FAKE, o=FAKE):
        return lib.hg_attn_partial_static(ctypes.byref(desc), packed, n, m, l, o, None)

    assert call(_desc([10], dtype=7)) == -3
    assert call(_desc([10], d=96)) == -2
    assert call(_desc([10]), packed=B.pack_ranges([(0, 0, 11)])) == -4
    assert call(_desc([10]), m=None) == -1
    assert lib.hg_attn_partial_static(None, None, 0, None, None, None, None) == -1
    assert call(_desc([10]), packed=None, n=0, m=None, l=None, o=None) == 0  # nothing to do
    # 64 KV heads x 2000 one-token ranges: 128k segment records of 520 bytes, far beyond 16 MiB
    many = [(0, i, i + 1) for i in range(2000)]
    big = _desc([100000], hq=64, hkv=64)
    sz = ctypes.c_size_t()
    pm = B.pack_ranges(many)
    assert lib.hg_attn_partial_workspace_size(ctypes.byref(big), pm, len(many), ctypes.byref(sz)) == 0
    assert sz.value > (16 << 20)
    assert call(big, packed=pm, n=len(many)) == -5


def test_partial_merge_validates_before_any_launch(lib):
    """hg_attn_partial_merge: the checks of both calls it stands for, on the host, before anything
    is enqueued (compute_units() is not asked for: without a GPU nothing may touch the runtime)."""
    good = B.pack_ranges([(0, 0, 10), (0, 10, 20)])
    gp = np.array([0, 2], dtype=np.int32)

    def call(desc, packed=good, n=2, groups=gp.ctypes.data, g=1, m=FAKE, l=FAKE, o=FAKE, out=FAKE, ws=FAKE * 16, ws_bytes=1 << 40):
        return lib.hg_attn_partial_merge(ctypes.byref(desc), packed, n, groups, g, m, l, o, out, None, ws, ws_bytes, None)

    assert call(_desc([20], dtype=7)) == -3
    assert call(_desc([20], d=96)) == -2
    assert call(_desc([20]), packed=B.pack_ranges([(0, 0, 10), (0, 10, 21)])) == -4
    assert call(_desc([20]), groups=None) == -1
    assert call(_desc([20]), groups=np.array([0, 1], dtype=np.int32).ctypes.data) == -4  # the groups must cover the ranges
    assert call(_desc([20]), groups=np.array([1, 2], dtype=np.int32).ctypes.data) == -4
    assert call(_desc([20]), out=None) == -1
    assert call(_desc([20]), m=None) == -1
    assert call(_desc([20]), g=70000) == -2
    sz = ctypes.c_size_t()
    assert lib.hg_attn_partial_merge_workspace_size(ctypes.byref(_desc([20])), good, 2, gp.ctypes.data, 1, ctypes.byref(sz)) == 0
    assert lib.hg_attn_partial_merge_workspace_size(ctypes.byref(_desc([20])), good, 2, gp.ctypes.data, 1, None) == -1
    big = _desc([5000000], hq=64, hkv=64)
    pm = B.pack_ranges([(0, 0, 5000000)])
    assert lib.hg_attn_partial_merge_workspace_size(ctypes.byref(big), pm, 1, np.array([0, 1], dtype=np.int32).ctypes.data, 1,
                                                    ctypes.byref(sz)) == 0
    assert sz.value > 4096
    assert lib.hg_attn_partial_merge(ctypes.byref(big), pm, 1, np.array([0, 1], dtype=np.int32).ctypes.data, 1, FAKE, FAKE, FAKE,
                                     FAKE, None, FAKE * 16, 64, None) == -5  # workspace too small
    assert call(_desc([20]), packed=None, n=0, groups=np.array([0], dtype=np.int32).ctypes.data, g=0, m=None, l=None, o=None,
                out=None) == 0  # nothing to do


def test_measurement_aids_validate_their_arguments(lib):
    assert lib.hg_attn_calibration_stream(None, 1 << 30, FAKE, 32, 1, 0, None) == -1
    assert lib.hg_attn_calibration_stream(FAKE, 1 << 30, None, 32, 1, 0, None) == -1   # writes need a destination
    assert lib.hg_attn_calibration_stream(FAKE + 4, 1 << 30, FAKE, 0, 1, 0, None) == -2  # misaligned
    assert lib.hg_attn_calibration_stream(FAKE, 1 << 30, FAKE, 4096, 1, 0, None) == -2
    assert lib.hg_attn_calibration_stream(FAKE, 1 << 30, FAKE, 32, 0, 0, None) == -2
    assert lib.hg_attn_calibration_stream(FAKE, 1000, FAKE, 0, 1, 0, None) == -2       # less than one iteration per workgroup
    assert lib.hg_attn_calibration_copy(None, FAKE, 16, None) == -1
    assert lib.hg_attn_calibration_copy(FAKE, FAKE * 2, 8, None) == -2
    assert lib.hg_attn_profile_start(-1, 1) == -2 and lib.hg_attn_profile_start(1, 0) == -2
    n = ctypes.c_int32(-1)
    assert lib.hg_attn_profile_times(None, 4, ctypes.byref(n)) == -1
    assert lib.hg_attn_profile_times(None, 0, ctypes.byref(n)) == 0 and n.value == 0


def test_strerror_is_total(lib):
    for code in range(-8, 2):
        assert isinstance(B.hg_strerror(code), str) and B.hg_strerror(code)
    assert B.hg_strerror(0) == "ok"


def _partial(lib, desc, ranges, m=FAKE, l=FAKE, o=FAKE, ws=FAKE * 16, ws_bytes=1 << 40):
    packed = B.pack_ranges(ranges)
    return lib.hg_attn_partial(ctypes.byref(desc), packed, len(ranges), m, l, o, ws, ws_bytes, None)


def test_partial_rejects_bad_arguments_before_any_launch(lib):
    good = [(0, 0, 10)]
    assert _partial(lib, _desc([10], dtype=7), good) == -3
    assert _partial(lib, _desc([10], d=96), good) == -2
    assert _partial(lib, _desc([10], hq=5, hkv=2), good) == -2
    assert _partial(lib, _desc([10], q=0), good) == -1
    assert _partial(lib, _desc([10], k=FAKE + 8), good) == -2  # misaligned base
    assert _partial(lib, _desc([10], stride_t=64), good) == -2  # rows overlap
    assert _partial(lib, _desc([10], stride_t=132), good) == -2  # rows not 16-byte aligned
    assert _partial(lib, _desc([10], stride_t=1 << 26), good) == -2  # rows 128 MiB apart: beyond 32-bit offsets
    assert _partial(lib, _desc([10], scale=float("nan")), good) == -2
    assert _partial(lib, _desc([-1]), good) == -4
    for bad in [(0, 5, 4), (0, 0, 11), (1, 0, 1), (-1, 0, 1), (0, -1, 3)]:
        assert _partial(lib, _desc([10]), [bad]) == -4
    assert _partial(lib, _desc([10]), good, m=None) == -1
    assert _partial(lib, _desc([10]), good, ws=None) == -5
    assert _partial(lib, _desc([10]), good, ws=FAKE + 16) == -5  # not 256-byte aligned
    assert _partial(lib, _desc([10]), good, ws_bytes=8) == -5
    assert lib.hg_attn_partial(None, None, 0, None, None, None, None, 0, None) == -1
    # nothing to do is fine and touches nothing
    assert _partial(lib, _desc([10]), [], m=None, l=None, o=None, ws=None, ws_bytes=0) == 0


def test_full_and_merge_reject_bad_arguments(lib):
    d = _desc([10, 20])
    assert lib.hg_attn_full(ctypes.byref(d), None, None, FAKE * 16, 1 << 40, None) == -1
    assert lib.hg_attn_full(ctypes.byref(d), FAKE, None, None, 0, None) == -5
    gp = np.array([0, 2, 1], dtype=np.int32)
    assert lib.hg_attn_merge(FAKE, FAKE, FAKE, gp.ctypes.data, 2, 4, 128, FAKE, None, None, 0, None) == -4
    gp = np.array([-1, 2], dtype=np.int32)
    assert lib.hg_attn_merge(FAKE, FAKE, FAKE, gp.ctypes.data, 1, 4, 128, FAKE, None, None, 0, None) == -4
    gp = np.array([0, 2], dtype=np.int32)
    assert lib.hg_attn_merge(FAKE, FAKE, FAKE, gp.ctypes.data, 1, 4, 100, FAKE, None, None, 0, None) == -2
    assert lib.hg_attn_merge(FAKE, FAKE, FAKE, gp.ctypes.data, 1, 4, 128, None, None, None, 0, None) == -1
    assert lib.hg_attn_merge(None, FAKE, FAKE, gp.ctypes.data, 1, 4, 128, FAKE, None, None, 0, None) == -1
    assert lib.hg_attn_merge(FAKE, FAKE, FAKE, None, 1, 4, 128, FAKE, None, None, 0, None) == -1
    assert lib.hg_attn_merge(None, None, None, None, 0, 4, 128, None, None, None, 0, None) == 0
    one = np.array([0, 1], dtype=np.int32)
    assert lib.hg_attn_merge2(FAKE, FAKE, FAKE, one.ctypes.data, FAKE, FAKE, FAKE, None, 1, 4, 128, FAKE, None, None, 0, None) == -1
    assert lib.hg_attn_merge2(FAKE, FAKE, FAKE, one.ctypes.data, None, FAKE, FAKE, one.ctypes.data, 1, 4, 128, FAKE, None, None, 0, None) == -1
    bad = np.array([1, 0], dtype=np.int32)
    assert lib.hg_attn_merge2(FAKE, FAKE, FAKE, one.ctypes.data, FAKE, FAKE, FAKE, bad.ctypes.data, 1, 4, 128, FAKE, None, None, 0, None) == -4
    big = np.arange(1000, dtype=np.int32)  # more groups than fit in kernel arguments: needs workspace
    sz = ctypes.c_size_t()
    assert lib.hg_attn_merge_workspace_size(999, ctypes.byref(sz)) == 0 and sz.value >= 4000
    assert lib.hg_attn_merge(FAKE, FAKE, FAKE, big.ctypes.data, 999, 4, 128, FAKE, None, None, 0, None) == -5


def test_topk_rejects_bad_arguments_before_any_launch(lib):
    d = _desc([1000, 20])
    packed = B.pack_ranges([(0, 0, 900), (1, 0, 20)])
    gp = np.array([0, 1, 2], dtype=np.int32)

    def call(desc=d, ranges=packed, n=2, groups=gp.ctypes.data, g=2, k=16, sel=FAKE, m=FAKE, l=FAKE, o=FAKE, ws=FAKE * 16,
             ws_bytes=1 << 40):
        return lib.hg_attn_topk(ctypes.byref(desc), ranges, n, groups, g, k, sel, m, l, o, ws, ws_bytes, None)

    assert call(k=0) == -2 and call(k=5000) == -2
    assert call(m=None) == -1 and call(groups=None) == -1
    assert call(ws=None, ws_bytes=0) == -5 and call(ws_bytes=64) == -5
    bad = np.array([0, 2, 1], dtype=np.int32)
    assert call(groups=bad.ctypes.data) == -4
    mixed = np.array([0, 2, 2], dtype=np.int32)  # a group may not span two sequences
    assert call(groups=mixed.ctypes.data) == -4
    assert call(ranges=B.pack_ranges([(0, 0, 1001), (1, 0, 20)])) == -4
    sz, sz2 = ctypes.c_size_t(), ctypes.c_size_t()
    assert lib.hg_attn_topk_workspace_size(ctypes.byref(d), packed, 2, gp.ctypes.data, 2, 16, ctypes.byref(sz)) == 0
    # room for every logit of every head at least (the two-call sequence inside keeps them there)
    assert sz.value >= 4 * 920 * 4
    try:
        assert lib.hg_attn_set_topk_mode(1) == 0
        assert lib.hg_attn_topk_workspace_size(ctypes.byref(d), packed, 2, gp.ctypes.data, 2, 16, ctypes.byref(sz2)) == 0
        assert sz2.value >= 2 * sz.value - 4096  # the scan's worst case: two such arrays (values and columns)
        assert lib.hg_attn_set_topk_mode(4) == -2 and lib.hg_attn_set_topk_mode(-1) == -2
    finally:
        lib.hg_attn_set_topk_mode(0)
    assert call(n=0, g=0, ranges=None, groups=gp.ctypes.data) == 0  # nothing to do


def test_gather_rejects_bad_arguments_before_any_launch(lib):
    d = _desc([10, 20])
    seqs = np.array([0, 1, 1], dtype=np.int32)

    def call(desc=d, gs=seqs.ctypes.data, n=3, index=FAKE, max_k=8, m=FAKE, l=FAKE, o=FAKE, ws=None, ws_bytes=0):
        return lib.hg_attn_gather(ctypes.byref(desc), gs, n, index, max_k, m, l, o, ws, ws_bytes, None)

    assert call(desc=_desc([10, 20], dtype=9)) == -3
    assert call(desc=_desc([10, 20], d=80)) == -2
    assert call(max_k=0) == -2 and call(max_k=(1 << 20) + 1) == -2 and call(n=-1) == -2 and call(n=70000) == -2
    assert call(index=None) == -1 and call(gs=None) == -1 and call(m=None) == -1 and call(o=None) == -1
    for bad in ([0, 2, 1], [-1, 0, 0]):
        b = np.array(bad, dtype=np.int32)
        assert call(gs=b.ctypes.data) == -4
    assert call(n=0, index=None, gs=None, m=None, l=None, o=None) == 0  # nothing to do
    many = np.zeros(1000, dtype=np.int32)
    sz = ctypes.c_size_t()
    assert lib.hg_attn_gather_workspace_size(1000, ctypes.byref(sz)) == 0 and sz.value >= 4000
    assert lib.hg_attn_gather_workspace_size(3, ctypes.byref(sz)) == 0 and sz.value == 0
    assert call(gs=many.ctypes.data, n=1000) == -5
    assert lib.hg_attn_gather_workspace_size(-1, ctypes.byref(sz)) == -2
    assert lib.hg_attn_gather_workspace_size(3, None) == -1


def _plan(lib, desc, ranges):
    packed = B.pack_ranges(ranges)
    tile, n = ctypes.c_int32(), ctypes.c_int64()
    st = lib.hg_attn_plan(ctypes.byref(desc), packed, len(ranges), ctypes.byref(tile), ctypes.byref(n))
    assert st == 0
    return tile.value, n.value


def test_span_plan_covers_the_work(lib):
    """Equal spans over the linear work space: streams x tokens-in-all-ranges positions."""
    try:
        seq = [5000, 70, 0, 1 << 20]
        ranges = [(0, 0, 5000), (0, 17, 17), (1, 3, 70), (3, 0, 1 << 20), (3, 1000, 1001), (0, 4999, 5000)]
        ltok = sum(e - b for _, b, e in ranges)
        streams = 2  # hkv = 2, both query heads of a KV head travel together
        for forced in (0, 64, 128, 1024, 4096, 1 << 20):
            assert lib.hg_attn_set_span_tokens(forced) == 0
            span, n = _plan(lib, _desc(seq), ranges)
            assert span % 64 == 0 and 64 <= span
            if forced:
                assert span == forced
            else:
                assert n <= 256  # one workgroup per compute unit (256 assumed without a GPU)
            assert n == (streams * ltok + span - 1) // span
        for bad in (63, 100, -64, (1 << 24) + 64):
            assert lib.hg_attn_set_span_tokens(bad) == -2
        # workspace holds one record of (d + 2) floats per head for every possible segment
        lib.hg_attn_set_span_tokens(64)
        d = _desc(seq)
        sz = ctypes.c_size_t()
        packed = B.pack_ranges(ranges)
        assert lib.hg_attn_partial_workspace_size(ctypes.byref(d), packed, len(ranges), ctypes.byref(sz)) == 0
        span, n = _plan(lib, d, ranges)
        assert sz.value >= (n + streams * len(ranges)) * 2 * (128 + 2) * 4
        # nothing to stream: no workgroups, and only empty ranges still plan fine
        span, n = _plan(lib, _desc(seq), [(0, 5, 5), (2, 0, 0)])
        assert n == 0
    finally:
        lib.hg_attn_set_span_tokens(0)


def test_large_range_tables_need_table_space(lib):
    seq = [100000]
    many = [(0, i, i + 1) for i in range(500)]
    d = _desc(seq)
    sz_many, sz_few = ctypes.c_size_t(), ctypes.c_size_t()
    pm, pf = B.pack_ranges(many), B.pack_ranges(many[:10])
    assert lib.hg_attn_partial_workspace_size(ctypes.byref(d), pm, 500, ctypes.byref(sz_many)) == 0
    assert lib.hg_attn_partial_workspace_size(ctypes.byref(d), pf, 10, ctypes.byref(sz_few)) == 0
    assert sz_many.value > sz_few.value

"""hg_attn_partial_static (the entry point that allocates nothing) against hg_attn_partial.

Two calls in a row on one stream share the library's static scratch buffer, the second with a
smaller input: whatever the first call left in the buffer must not leak into the second result.
Both calls must match the existing entry point (same kernels, same plan: bit for bit) and the
oracle to the usual bars.
"""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2604_18529_amd as hg
from paper_2604_18529_amd import hg_attn as B
from paper_2604_18529_amd import workloads as W

from parity_utils import check_out, check_triples, kv_np, to_np

pytestmark = pytest.mark.gpu

BIG = W.WorkloadSpec("static-big", 3, 16, 4, 128, "f16", 20000, 40000, "dirichlet", 5, outlier_k=True, seed=21)
SMALL = W.WorkloadSpec("static-small", 1, 16, 4, 128, "f16", 700, 700, "ratios", 3, seed=22)
BIG_MHA = W.WorkloadSpec("static-big-mha", 2, 6, 6, 64, "f32", 9000, 12000, "dirichlet", 4, seed=23)
SMALL_MHA = W.WorkloadSpec("static-small-mha", 1, 6, 6, 64, "f32", 130, 130, "half", 2, seed=24)


def _static_through_c_abi(w):
    """The C call itself: descriptor, host range table, caller-owned outputs, stream; no workspace."""
    lib = hg.load_library()
    desc, keep = B.make_desc(w.q, w.k, w.v, w.seq_lens, w.scale)
    packed = B.pack_ranges(w.ranges)
    R, Hq, d = len(w.ranges), w.q.shape[1], w.q.shape[2]
    m = torch.full((R, Hq), float("nan"), dtype=torch.float32, device=w.q.device)
    l = torch.full((R, Hq), float("nan"), dtype=torch.float32, device=w.q.device)
    o = torch.full((R, Hq, d), float("nan"), dtype=torch.float32, device=w.q.device)
    stream = torch.cuda.current_stream().cuda_stream or None
    st = lib.hg_attn_partial_static(ctypes.byref(desc), packed, R, m.data_ptr(), l.data_ptr(), o.data_ptr(), stream)
    assert st == 0, B.hg_strerror(st)
    del keep
    return m, l, o


@pytest.mark.parametrize("big,small", [(BIG, SMALL), (BIG_MHA, SMALL_MHA)], ids=["gqa-f16-d128", "mha-f32-d64"])
def test_static_scratch_matches_partial_twice_in_a_row(big, small):
    wb, ws = W.make_workload(big, "cuda:0"), W.make_workload(small, "cuda:0")
    # both static calls first, back to back on one stream; the references afterwards
    got_b = _static_through_c_abi(wb)
    got_s = _static_through_c_abi(ws)
    torch.cuda.synchronize()
    for w, got, what in ((wb, got_b, "first call"), (ws, got_s, "second, smaller call")):
        ref = hg.hg_attn_partial(w.q, w.k, w.v, w.seq_lens, w.ranges, w.scale)
        torch.cuda.synchronize()
        for a, b, name in zip(got, ref, "mlo"):
            assert torch.equal(a, b), "%s: %s differs from hg_attn_partial" % (what, name)
        kn, vn = kv_np(w)
        mo, lo, oo = oracle.attn_partial(to_np(w.q), kn, vn, w.seq_lens, w.scale, w.ranges)
        check_triples(*got, mo, lo, oo, what)
        out, lse = hg.hg_attn_merge(*got, w.group_ptr)
        ref_out, ref_lse = oracle.attn_full(to_np(w.q), kn, vn, w.seq_lens, w.scale)
        check_out(out, lse, ref_out, ref_lse, what + " merged")


def test_static_scratch_refuses_what_does_not_fit():
    """More segment records than the static buffer holds: a clear error, outputs untouched."""
    spec = W.WorkloadSpec("static-too-big", 1, 64, 64, 64, "f16", 4096, 4096, "none", 1, seed=25)
    w = W.make_workload(spec, "cuda:0")
    ranges = [(0, i, i + 1) for i in range(2000)]
    lib = hg.load_library()
    desc, keep = B.make_desc(w.q, w.k, w.v, w.seq_lens, w.scale)
    packed = B.pack_ranges(ranges)
    m = torch.full((len(ranges), 64), 7.0, dtype=torch.float32, device="cuda:0")
    l, o = m.clone(), torch.full((len(ranges), 64, 64), 7.0, dtype=torch.float32, device="cuda:0")
    st = lib.hg_attn_partial_static(ctypes.byref(desc), packed, len(ranges), m.data_ptr(), l.data_ptr(), o.data_ptr(), None)
    torch.cuda.synchronize()
    assert st == -5
    assert bool((m == 7.0).all()) and bool((l == 7.0).all()) and bool((o == 7.0).all())
    # the same problem through the workspace entry point works
    got = hg.hg_attn_partial(w.q, w.k, w.v, w.seq_lens, ranges, w.scale)
    mo, lo, oo = oracle.attn_partial(to_np(w.q), *kv_np(w), w.seq_lens, w.scale, ranges)
    check_triples(*got, mo, lo, oo, "workspace entry point")
    del keep

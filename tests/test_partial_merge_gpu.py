"""hg_attn_partial_merge: hg_attn_partial and hg_attn_merge in one call.

Small inputs take the one-launch path (one workgroup per (group, stream) streams the group's
ranges, writes their triples and the merged output); everything else runs the two calls'
kernels.  Either way the triples must equal hg_attn_partial's to the usual bars against the
oracle, and the merged output hg_attn_merge's."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_18529_amd as hg
from paper_2604_18529_amd import workloads as W

from parity_utils import check_out, check_triples, kv_np, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _check(w, ranges, gp, what, expect_same_triples=True):
    m, l, o, out, lse = hg.hg_attn_partial_merge(w.q, w.k, w.v, w.seq_lens, ranges, gp, w.scale)
    m2, l2, o2 = hg.hg_attn_partial(w.q, w.k, w.v, w.seq_lens, ranges, w.scale)
    out2, lse2 = hg.hg_attn_merge(m2, l2, o2, gp)
    torch.cuda.synchronize()
    kn, vn = kv_np(w)
    mo, lo, oo = oracle.attn_partial(to_np(w.q), kn, vn, w.seq_lens, w.scale, ranges)
    check_triples(m, l, o, mo, lo, oo, what)
    # the oracle's merge of its own triples, group by group
    ref, rlse = oracle.attn_merge(mo, lo, oo, gp)
    check_out(out, lse, ref, rlse, what + " merged")
    assert (out - out2).abs().max().item() <= 2e-5, what
    both = torch.isfinite(lse2)
    assert torch.equal(torch.isfinite(lse), both) and (lse[both] - lse2[both]).abs().max().item() <= 2e-5, what


# (dtype, head_dim, query heads, KV heads): the vector kernel with 1, 2, 4 and 8 heads per stream
SMALL = [("f32", 64, 4, 4), ("f32", 128, 4, 2), ("f32", 64, 12, 3), ("f32", 128, 8, 1), ("f16", 128, 6, 6), ("bf16", 64, 3, 3),
         ("f16", 64, 5, 5)]


@pytest.mark.parametrize("dtype,d,hq,hkv", SMALL)
def test_small_inputs_in_one_launch(dtype, d, hq, hkv):
    """The tiny benchmark shape and its like: ragged ranges, an empty range, a group of one range,
    a group without tokens."""
    spec = W.WorkloadSpec("pm-small", 3, hq, hkv, d, dtype, 40, 300, "none", seed=140 + hq)
    w = W.make_workload(spec, DEV)
    n = [int(x) for x in w.seq_lens]
    ranges = [(0, 0, n[0] // 3), (0, n[0] // 3, n[0] // 3), (0, n[0] // 3, n[0]), (1, 0, n[1]), (2, 5, 5)]
    gp = [0, 3, 4, 5]
    _check(w, ranges, gp, "%s d=%d %d/%d" % (dtype, d, hq, hkv))


def test_tiny_benchmark_shape():
    w = W.make_workload(W.WORKLOADS[0], DEV)
    _check(w, w.ranges, w.group_ptr, W.WORKLOADS[0].name)


@pytest.mark.parametrize("case", ["long", "many-groups", "gqa", "paged", "many-ranges"])
def test_everything_else_runs_the_two_calls_kernels(case):
    if case == "long":
        spec = W.WorkloadSpec("pm-long", 2, 4, 4, 128, "f16", 3000, 5000, "dirichlet", 3, seed=150)
    elif case == "many-groups":
        spec = W.WorkloadSpec("pm-groups", 40, 2, 2, 64, "f32", 30, 90, "half", 2, seed=151)
    elif case == "gqa":
        spec = W.WorkloadSpec("pm-gqa", 2, 8, 2, 128, "f16", 100, 400, "half", 2, seed=152)
    elif case == "paged":
        spec = W.WorkloadSpec("pm-paged", 2, 4, 4, 64, "f16", 100, 300, "half", 2, seed=153)
    else:
        spec = W.WorkloadSpec("pm-ranges", 1, 4, 4, 64, "f32", 700, 700, "none", seed=154)
    w = W.make_workload(spec, DEV)
    ranges, gp = w.ranges, w.group_ptr
    if case == "many-ranges":
        ranges = [(0, 7 * i, 7 * i + 7) for i in range(100)]
        gp = [0, 100]
    if case == "paged":
        k_p, v_p, table = W.make_paged(w, 16, seed=5)
        m, l, o, out, lse = hg.hg_attn_partial_merge(w.q, k_p, v_p, w.seq_lens, ranges, gp, w.scale, block_table=table)
        kn, vn = kv_np(w)
        mo, lo, oo = oracle.attn_partial(to_np(w.q), kn, vn, w.seq_lens, w.scale, ranges)
        check_triples(m, l, o, mo, lo, oo, case)
        ref, rlse = oracle.attn_merge(mo, lo, oo, gp)
        check_out(out, lse, ref, rlse, case + " merged")
        return
    _check(w, ranges, gp, case)


def test_merged_output_equals_unsplit_attention():
    """Ranges that tile every sequence once: the merged output is attention over the whole cache."""
    spec = W.WorkloadSpec("pm-tile", 2, 4, 4, 64, "f32", 200, 420, "dirichlet", 4, seed=155)
    w = W.make_workload(spec, DEV)
    m, l, o, out, lse = hg.hg_attn_partial_merge(w.q, w.k, w.v, w.seq_lens, w.ranges, w.group_ptr, w.scale)
    ref, rlse = oracle.attn_full(to_np(w.q), *kv_np(w), w.seq_lens, w.scale)
    check_out(out, lse, ref, rlse, "tiling ranges")


def test_which_inputs_take_the_one_launch_path():
    """The library's kernel-timing aid counts the calls that launch the ordinary streaming kernel
    (hg_attn_partial's); a call that takes the one-launch path does not."""
    small = W.make_workload(W.WORKLOADS[0], DEV)
    long_ = W.make_workload(W.WorkloadSpec("pm-long", 2, 4, 4, 128, "f16", 3000, 5000, "dirichlet", 3, seed=150), DEV)
    gqa = W.make_workload(W.WorkloadSpec("pm-gqa", 2, 8, 2, 128, "f16", 100, 400, "half", 2, seed=152), DEV)
    for w, want in ((small, 0), (long_, 1), (gqa, 1)):
        hg.hg_attn_profile_start(4, 1)
        try:
            hg.hg_attn_partial_merge(w.q, w.k, w.v, w.seq_lens, w.ranges, w.group_ptr, w.scale)
            torch.cuda.synchronize()
        finally:
            _, launches = hg.hg_attn_profile_stop()
        assert launches == want, w.spec.name

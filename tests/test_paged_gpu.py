"""Paged KV caches (block table + physical block pool): every entry point must give what the
oracle gives on the equivalent contiguous cache, for every kernel variant, with blocks in shuffled
physical order and ragged tails."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_18529_amd as hg
from paper_2604_18529_amd import workloads as W

from parity_utils import check_out, check_triples, kv_np, to_np
from test_concat_gpu import LOGIT_TOL, _oracle_concat

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(autouse=True)
def _default_spans():
    hg.hg_attn_set_span_tokens(0)
    yield
    hg.hg_attn_set_span_tokens(0)


def _run_paged(w, block_tokens, what, ranges=None, gp=None, routes=True):
    ranges = w.ranges if ranges is None else ranges
    gp = w.group_ptr if gp is None else gp
    kp, vp, table = W.make_paged(w, block_tokens, seed=3)
    m, l, o = hg.hg_attn_partial(w.q, kp, vp, w.seq_lens, ranges, w.scale, block_table=table)
    qn = to_np(w.q)
    kn, vn = kv_np(w)
    mo, lo, oo = oracle.attn_partial(qn, kn, vn, w.seq_lens, w.scale, ranges)
    check_triples(m, l, o, mo, lo, oo, what + " partial")
    out, lse = hg.hg_attn_merge(m, l, o, gp)
    ref, rlse = oracle.attn_merge(mo, lo, oo, gp)
    check_out(out, lse, ref, rlse, what + " merge")
    fout, flse = hg.hg_attn_full(w.q, kp, vp, w.seq_lens, w.scale, block_table=table)
    fref, frlse = oracle.attn_full(qn, kn, vn, w.seq_lens, w.scale)
    check_out(fout, flse, fref, frlse, what + " full")
    # logits export, the paper-literal concat and the Post-QK^T selection through the same table
    lg = hg.hg_attn_logits(w.q, kp, vp, w.seq_lens, ranges, w.scale, block_table=table)
    lg_ref = oracle.attn_logits(qn, kn, vn, w.seq_lens, w.scale, ranges)
    if lg_ref.size:
        assert np.abs(to_np(lg).astype(np.float64) - lg_ref).max() <= LOGIT_TOL, what + " logits"
    if not routes:  # the caller's groups mix sequences, which concat and select do not take
        return kp, vp, table
    cout, clse = hg.hg_attn_concat(w.q, kp, vp, w.seq_lens, ranges, lg, gp, w.scale, block_table=table)
    cref, crlse = _oracle_concat(w, ranges, gp)
    check_out(cout, clse, cref, crlse, what + " concat")
    lg_np = to_np(lg)
    sel, sm, sl, so = hg.hg_attn_select(w.q, kp, vp, w.seq_lens, ranges, lg, gp, 40, w.scale, block_table=table)
    rsel, rm, rl, ro = oracle.attn_select(qn, kn, vn, w.seq_lens, w.scale, ranges, lg_np, gp, 40)
    assert np.array_equal(to_np(sel), rsel), what + " select: kept tokens differ"
    check_triples(sm, sl, so, rm, rl, ro, what + " select")
    return kp, vp, table


@pytest.mark.parametrize("block_tokens", [16, 64, 1024])
@pytest.mark.parametrize("dtype,d,group", [("f16", 128, 1), ("f16", 128, 8), ("f32", 64, 1), ("f16", 64, 2), ("f32", 128, 4),
                                            ("f16", 128, 16), ("f16", 128, 5), ("f16", 64, 4), ("f16", 64, 9), ("bf16", 128, 4), ("bf16", 64, 1), ("bf16", 64, 6)])
def test_paged_matches_contiguous(dtype, d, group, block_tokens):
    spec = W.WorkloadSpec("paged", 3, 2 * group, 2, d, dtype, 1, 3000, "ratios", 3, seed=70 + group)
    w = W.make_workload(spec, DEV)
    _run_paged(w, block_tokens, "%s d=%d G=%d bt=%d" % (dtype, d, group, block_tokens))


@pytest.mark.parametrize("span", [64, 256])
def test_paged_small_spans_and_edge_ranges(span):
    hg.hg_attn_set_span_tokens(span)
    spec = W.WorkloadSpec("pagededge", 3, 8, 1, 128, "f16", 0, 1000, "none", seed=71)
    w = W.make_workload(spec, DEV)
    w.seq_lens[:] = [1000, 0, 17]
    ranges = [(0, 0, 0), (0, 15, 17), (0, 16, 16), (0, 0, 1000), (2, 0, 17), (2, 16, 17), (0, 999, 1000), (0, 31, 33)]
    _run_paged(w, 16, "edge span=%d" % span, ranges, [0, 4, 4, 8], routes=False)
    # the same edge ranges grouped per sequence, for the routes that need one sequence per group
    ranges = [(0, 0, 0), (0, 15, 17), (0, 16, 16), (0, 0, 1000), (0, 999, 1000), (0, 31, 33), (2, 0, 17), (2, 16, 17)]
    _run_paged(w, 16, "edge groups span=%d" % span, ranges, [0, 6, 6, 8])


def test_zero_query_bitplanes_are_exact_through_the_block_table():
    """q = 0 and bit-plane values: l and O are exact integers, which pins that every token was
    fetched from the right physical block and row."""
    hg.hg_attn_set_span_tokens(128)
    N, d = 5000, 128
    spec = W.WorkloadSpec("pagedbits", 1, 8, 1, d, "f16", N, N, "none", seed=72)
    w = W.make_workload(spec, DEV)
    w.q.zero_()
    w.v[0, 0] = W.bitplane_values(N, d, torch.float16, DEV)
    kp, vp, table = W.make_paged(w, 16, seed=4)
    ranges = [(0, 0, N), (0, 1, 4999), (0, 15, 17), (0, 16, 32), (0, 1000, 1001)] + W.random_ranges([N], 30, seed=5)
    m, l, o = hg.hg_attn_partial(w.q, kp, vp, w.seq_lens, ranges, w.scale, block_table=table)
    mo, lo, oo = oracle.attn_partial(to_np(w.q), *kv_np(w), w.seq_lens, w.scale, ranges)
    assert np.array_equal(to_np(l).astype(np.float64), lo)
    assert np.array_equal(to_np(o).astype(np.float64), oo)


def test_short_block_table_is_rejected():
    spec = W.WorkloadSpec("pagedrej", 1, 2, 2, 64, "f16", 100, 100, "none", seed=73)
    w = W.make_workload(spec, DEV)
    kp, vp, table = W.make_paged(w, 16)
    # a table that is too short for a sequence is caught on the host
    short = table[:, :3].contiguous()
    with pytest.raises(hg.HgError) as ei:
        hg.hg_attn_full(w.q, kp, vp, w.seq_lens, w.scale, block_table=short)
    assert ei.value.status == -4


@pytest.mark.parametrize("index,block_tokens", [(1, 16), (4, 256)])
def test_paged_full_size(index, block_tokens):
    """Benchmark shapes through a shuffled block pool: equal to the contiguous result (both on the
    GPU, which the contiguous tests tie to the oracle) and sampled pairs against the oracle."""
    spec = W.WORKLOADS[index]
    w = W.make_workload(spec, DEV)
    kp, vp, table = W.make_paged(w, block_tokens, seed=6)
    m, l, o = hg.hg_attn_partial(w.q, kp, vp, w.seq_lens, w.ranges, w.scale, block_table=table)
    out, lse = hg.hg_attn_merge(m, l, o, w.group_ptr)
    cout, clse = hg.hg_attn_full(w.q, w.k, w.v, w.seq_lens, w.scale)
    assert (out - cout).abs().max().item() <= 2e-5 and (lse - clse).abs().max().item() <= 2e-5
    G = spec.n_q_heads // spec.n_kv_heads
    for b, h in [(0, 0), (spec.batch - 1, spec.n_q_heads - 1)]:
        n = int(w.seq_lens[b])
        ref, rlse = oracle.attn_full(to_np(w.q[b:b + 1, h:h + 1]), to_np(w.k[b:b + 1, h // G:h // G + 1, :n]),
                                     to_np(w.v[b:b + 1, h // G:h // G + 1, :n]), [n], w.scale)
        assert np.abs(to_np(out[b, h]) - ref[0, 0]).max() <= 2e-3 and abs(float(lse[b, h]) - rlse[0, 0]) <= 1e-3

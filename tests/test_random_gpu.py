"""Seeded random sweep over storage type, head size, query group, layout, paging, span length and
range tables: every entry point against the oracle.  The fixed cases of the other files pin the
known edges; this one looks for the combinations nobody thought of."""
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


def _grouped_ranges(rng, seq_lens, max_per_seq):
    """Ranges grouped by sequence (ascending, possibly overlapping, possibly empty) and their CSR."""
    ranges, gp = [], [0]
    for b, n in enumerate(seq_lens):
        k = int(rng.integers(0, max_per_seq + 1))
        rs = []
        for _ in range(k):
            a, c = sorted(int(x) for x in rng.integers(0, n + 1, size=2))
            if rng.random() < 0.15:
                c = a  # empty
            if rng.random() < 0.15:
                a, c = 0, int(n)  # the whole sequence
            rs.append((b, a, c))
        rs.sort(key=lambda r: (r[1], r[2]))
        ranges += rs
        gp.append(len(ranges))
    return ranges, gp


@pytest.mark.parametrize("case", list(range(96)) + list(range(100, 148)) + list(range(500, 532)))
def test_random_case(case):
    """Cases below 500 are short (every code path of a workgroup, many combinations; bf16 joins
    from case 100 on); cases from 500 are long enough for several spans per stream and for the two-stage selection."""
    rng = np.random.default_rng(1000 + case)
    big = case >= 500
    dtype = ["f16", "f32", "bf16"][int(rng.integers(2)) if case < 96 else case % 3]  # (the first 96 keep their draws)
    d = [64, 128][int(rng.integers(2))]
    group = int(rng.choice([1, 4, 8, 3] if big else [1, 1, 2, 3, 4, 6, 8, 16, 17]))
    hkv = int(rng.integers(1, 3 if big else 4))
    batch = int(rng.integers(1, 3 if big else 5))
    n_max = int(rng.choice([20000, 70000] if big else [40, 300, 1500, 4000]))
    layout = ["bhtd", "bthd"][int(rng.integers(2))]
    paged = rng.random() < 0.4
    block_tokens = int(rng.choice([16, 32, 128]))
    span = int(rng.choice([0, 0, 0, 4096] if big else [0, 0, 64, 192, 1024]))
    top_k = int(rng.choice([64, 256, 700] if big else [1, 5, 64, 200, 300, 1500]))
    what = "case %d: %s d=%d G=%d Hkv=%d B=%d n<=%d %s paged=%s/%d span=%d k=%d" % (
        case, dtype, d, group, hkv, batch, n_max, layout, paged, block_tokens, span, top_k)
    print(what, flush=True)

    spec = W.WorkloadSpec("rnd", batch, group * hkv, hkv, d, dtype, 0, n_max, "none", seed=2000 + case)
    w = W.make_workload(spec, DEV, layout=layout)
    if rng.random() < 0.3:
        w.seq_lens[int(rng.integers(batch))] = 0
    ranges, gp = _grouped_ranges(rng, w.seq_lens, 5)
    hg.hg_attn_set_span_tokens(span)
    qn = to_np(w.q)
    kn, vn = kv_np(w)
    if paged:
        k_dev, v_dev, table = W.make_paged(w, block_tokens, seed=case)
    else:
        k_dev, v_dev, table = w.k, w.v, None

    m, l, o = hg.hg_attn_partial(w.q, k_dev, v_dev, w.seq_lens, ranges, w.scale, block_table=table)
    mo, lo, oo = oracle.attn_partial(qn, kn, vn, w.seq_lens, w.scale, ranges)
    check_triples(m, l, o, mo, lo, oo, what + " partial")
    out, lse = hg.hg_attn_merge(m, l, o, gp)
    ref, rlse = oracle.attn_merge(mo, lo, oo, gp)
    check_out(out, lse, ref, rlse, what + " merge")
    pm, pl, po, pout, plse = hg.hg_attn_partial_merge(w.q, k_dev, v_dev, w.seq_lens, ranges, gp, w.scale, block_table=table)
    check_triples(pm, pl, po, mo, lo, oo, what + " partial_merge triples")
    check_out(pout, plse, ref, rlse, what + " partial_merge")
    fout, flse = hg.hg_attn_full(w.q, k_dev, v_dev, w.seq_lens, w.scale, block_table=table)
    fref, frlse = oracle.attn_full(qn, kn, vn, w.seq_lens, w.scale)
    check_out(fout, flse, fref, frlse, what + " full")

    lg = hg.hg_attn_logits(w.q, k_dev, v_dev, w.seq_lens, ranges, w.scale, block_table=table)
    lg_ref = oracle.attn_logits(qn, kn, vn, w.seq_lens, w.scale, ranges)
    assert lg.shape == lg_ref.shape
    if lg_ref.size:
        assert np.abs(to_np(lg).astype(np.float64) - lg_ref).max() <= LOGIT_TOL, what + " logits"
    cout, clse = hg.hg_attn_concat(w.q, k_dev, v_dev, w.seq_lens, ranges, lg, gp, w.scale, block_table=table)
    cref, crlse = _oracle_concat(w, ranges, gp)
    check_out(cout, clse, cref, crlse, what + " concat")

    # selection decides on the logits as given: quantise a copy so that ties occur
    lg_q = (torch.round(lg * 4) / 4).contiguous()
    sel, sm, sl, so = hg.hg_attn_select(w.q, k_dev, v_dev, w.seq_lens, ranges, lg_q, gp, top_k, w.scale, block_table=table)
    rsel, rm, rl, ro = oracle.attn_select(qn, kn, vn, w.seq_lens, w.scale, ranges, to_np(lg_q), gp, top_k)
    got = to_np(sel)
    if not np.array_equal(got, rsel):
        g, h = [int(x[0]) for x in np.nonzero((got != rsel).any(axis=2))]
        pre = np.cumsum([0] + [e - s for _, s, e in ranges])
        row = to_np(lg_q)[h, pre[gp[g]]:pre[gp[g + 1]]]
        raise AssertionError("%s select: kept tokens differ in group %d head %d\n got  %s\n want %s\n logits %s" % (
            what, g, h, got[g, h].tolist(), rsel[g, h].tolist(), row.tolist()))
    check_triples(sm, sl, so, rm, rl, ro, what + " select")

    # the one-call executor stage: the same kept tokens as logits -> select on the logits the library
    # itself computes (filtering scan forced on two cases of three, where it exists: once with the
    # one-launch selection behind it, once with the staged one), and the triple of the oracle's
    # listed-token routine over that list
    hg.hg_attn_set_topk_mode((1, 3, 0)[case % 3])
    try:
        tsel, tm, tl, to = hg.hg_attn_topk(w.q, k_dev, v_dev, w.seq_lens, ranges, gp, top_k, w.scale, block_table=table)
    finally:
        hg.hg_attn_set_topk_mode(0)
    usel, um, ul, uo = hg.hg_attn_select(w.q, k_dev, v_dev, w.seq_lens, ranges, lg, gp, top_k, w.scale, block_table=table)
    assert torch.equal(tsel, usel), what + " topk: kept tokens differ from logits -> select"
    tm3, tl3, to3 = oracle.attn_gather(qn, kn, vn, w.seq_lens, w.scale, list(range(batch)), to_np(tsel))
    check_triples(tm, tl, to, tm3, tl3, to3, what + " topk")

    # the kept lists evaluated again as listed tokens (true query), plus a list with padding and
    # duplicates at seeded positions; groups are the sequences that have a group of ranges
    group_seq = [b for b in range(batch)]
    rm2, rl2, ro2 = oracle.attn_gather(qn, kn, vn, w.seq_lens, w.scale, group_seq, rsel)
    gm, gl, go = hg.hg_attn_gather(w.q, k_dev, v_dev, w.seq_lens, group_seq, sel, w.scale, block_table=table)
    check_triples(gm, gl, go, rm2, rl2, ro2, what + " gather(sel)")
    max_k = int(rng.choice([1, 9, 70, 333]))
    idx = np.full((batch, group * hkv, max_k), -1, dtype=np.int32)
    for b in range(batch):
        n = int(w.seq_lens[b])
        if n:
            idx[b] = rng.integers(-n // 3 - 1, n, size=(group * hkv, max_k))  # about a quarter negative: padding
    rm3, rl3, ro3 = oracle.attn_gather(qn, kn, vn, w.seq_lens, w.scale, group_seq, idx)
    gm, gl, go = hg.hg_attn_gather(w.q, k_dev, v_dev, w.seq_lens, group_seq, torch.from_numpy(idx).to(DEV), w.scale,
                                   block_table=table)
    check_triples(gm, gl, go, rm3, rl3, ro3, what + " gather(random list)")

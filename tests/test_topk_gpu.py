"""GPU parity of hg_attn_topk, the Post-QK^T executor stage in one call: logits, top_k per (group,
head), kept tokens folded with their V rows -- with the logits never written out where the fused
scan applies.

Which tokens are kept is decided on fp32 logits.  The tests therefore compare
  * bit for bit against the oracle where every logit is exactly representable (dyadic q and K,
    power-of-two scale): both sides then decide on identical numbers, ties included;
  * bit for bit against hg_attn_logits -> hg_attn_select on ordinary data (that pair is tied to
    the oracle by its own tests, and the fused scan must reproduce it exactly);
  * against the oracle on ordinary data up to what rounding leaves open: every kept token's exact
    logit reaches the exact k-th largest within a tolerance, nothing clearly above it is missing,
    and the triple equals the oracle's listed-token routine over the kept list."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_18529_amd as hg
from paper_2604_18529_amd import workloads as W

from parity_utils import check_out, check_triples, kv_np, to_np
from test_concat_gpu import LOGIT_TOL

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(autouse=True, params=["scan", "scan-staged", "auto"])
def _modes(request):
    """Every test runs with the filtering scan forced wherever it exists (the inputs here are far
    shorter than what the library would choose it for) -- once with the one-launch selection from
    the scan's own lists behind it, once with the compaction and the staged selection that the
    library falls back to when those lists do not fit -- and with the library's own choice."""
    hg.hg_attn_set_span_tokens(0)
    hg.hg_attn_set_topk_mode({"scan": 1, "scan-staged": 3, "auto": 0}[request.param])
    yield
    hg.hg_attn_set_span_tokens(0)
    hg.hg_attn_set_topk_mode(0)


def _groups_per_sequence(w, rng, max_ranges=3, frac=0.8):
    """Offloaded ranges: per sequence up to max_ranges pieces of its first `frac` tokens
    (possibly empty, possibly with gaps), one group per sequence."""
    ranges, gp = [], [0]
    for b, n in enumerate(int(x) for x in w.seq_lens):
        hi = int(frac * n)
        cuts = sorted(int(x) for x in rng.integers(0, hi + 1, size=2 * int(rng.integers(1, max_ranges + 1))))
        for i in range(0, len(cuts), 2):
            ranges.append((b, cuts[i], cuts[i + 1]))
        gp.append(len(ranges))
    return ranges, gp


def _check_exact(w, ranges, gp, top_k, what):
    sel, m, l, o = hg.hg_attn_topk(w.q, w.k, w.v, w.seq_lens, ranges, gp, top_k, w.scale)
    rsel, rm, rl, ro, _ = oracle.attn_topk(to_np(w.q), *kv_np(w), w.seq_lens, w.scale, ranges, gp, top_k)
    got = to_np(sel)
    if not np.array_equal(got, rsel):
        g, h = [int(x[0]) for x in np.nonzero((got != rsel).any(axis=2))]
        raise AssertionError("%s: kept tokens differ in group %d head %d\n got  %s\n want %s" % (
            what, g, h, got[g, h].tolist(), rsel[g, h].tolist()))
    fin = np.isfinite(rm)
    assert np.array_equal(to_np(m).astype(np.float64)[fin], rm[fin]), what + ": m must be the kept maximum exactly"
    check_triples(m, l, o, rm, rl, ro, what)


# (dtype, d, query heads per KV head): the first rows take the fused scan, the others the
# two-call sequence inside the library
VARIANTS = [("f16", 128, 8), ("bf16", 128, 4), ("f16", 128, 2), ("f16", 128, 16), ("f16", 128, 5), ("f16", 128, 20),
            ("f16", 128, 1), ("f32", 64, 1), ("f16", 64, 4), ("f32", 128, 3), ("bf16", 64, 1)]


@pytest.mark.parametrize("top_k", [1, 64, 65, 128, 129, 256, 300])
@pytest.mark.parametrize("dtype,d,group", VARIANTS)
def test_bit_exact_on_exactly_representable_logits(dtype, d, group, top_k):
    spec = W.WorkloadSpec("topk", 3, 2 * group, 2, d, dtype, 200, 5000, "none", seed=110 + group)
    w = W.make_workload(spec, DEV)
    W.make_dyadic_(w, seed=111)
    w.scale = 0.125
    rng = np.random.default_rng(112 + top_k)
    ranges, gp = _groups_per_sequence(w, rng)
    _check_exact(w, ranges, gp, top_k, "%s d=%d G=%d k=%d" % (dtype, d, group, top_k))


@pytest.mark.parametrize("block_tokens", [16, 256])
@pytest.mark.parametrize("span", [0, 512])
@pytest.mark.parametrize("dtype,d,group", [("f16", 128, 8), ("bf16", 128, 2), ("f16", 128, 1), ("f32", 64, 1), ("bf16", 64, 1), ("f16", 64, 4)])
def test_paged_cache(dtype, d, group, span, block_tokens):
    """The same through a block table with physical blocks in shuffled order."""
    hg.hg_attn_set_span_tokens(span)
    spec = W.WorkloadSpec("topkpaged", 3, 2 * group, 2, d, dtype, 100, 6000, "none", seed=122 + group)
    w = W.make_workload(spec, DEV)
    W.make_dyadic_(w, seed=123)
    w.scale = 0.125
    kp, vp, table = W.make_paged(w, block_tokens, seed=9)
    rng = np.random.default_rng(124)
    ranges, gp = _groups_per_sequence(w, rng)
    for top_k in (40, 200):
        sel, m, l, o = hg.hg_attn_topk(w.q, kp, vp, w.seq_lens, ranges, gp, top_k, w.scale, block_table=table)
        rsel, rm, rl, ro, _ = oracle.attn_topk(to_np(w.q), *kv_np(w), w.seq_lens, w.scale, ranges, gp, top_k)
        assert np.array_equal(to_np(sel), rsel), "paged %s d=%d G=%d k=%d: kept tokens differ" % (dtype, d, group, top_k)
        check_triples(m, l, o, rm, rl, ro, "paged topk")


@pytest.mark.parametrize("span", [64, 192, 1024, 0])
@pytest.mark.parametrize("top_k", [3, 128, 200])
def test_many_segments_and_edge_ranges(span, top_k):
    """Forced short spans cut every range into many segments (and those into sub-spans with ragged
    tails); empty ranges, one-token ranges and an empty sequence are in the table."""
    hg.hg_attn_set_span_tokens(span)
    spec = W.WorkloadSpec("topkedge", 4, 16, 2, 128, "f16", 0, 3000, "none", seed=113)
    w = W.make_workload(spec, DEV)
    W.make_dyadic_(w, seed=114)
    w.scale = 0.125
    w.seq_lens[:] = [3000, 0, 77, 1500]
    ranges = [(0, 0, 0), (0, 5, 6), (0, 6, 1000), (0, 1000, 1000), (0, 1031, 2999), (2, 0, 77), (3, 100, 163), (3, 163, 1500)]
    gp = [0, 5, 5, 6, 8]
    _check_exact(w, ranges, gp, top_k, "span=%d k=%d" % (span, top_k))


@pytest.mark.parametrize("span", [256, 1024, 4096])
@pytest.mark.parametrize("dtype,group,top_k", [("f16", 8, 128), ("bf16", 4, 256), ("f16", 16, 7), ("f16", 2, 200), ("f16", 20, 100), ("bf16", 5, 64)])
def test_many_workgroups_per_group_share_their_bounds(dtype, group, top_k, span):
    """Long groups cut into many spans: the workgroups of a (range, stream) pair exchange bounds
    through memory while they run.  Whatever each of them happens to read, the kept set is the
    oracle's, bit for bit (run twice: the timing differs, the result must not)."""
    hg.hg_attn_set_span_tokens(span)
    spec = W.WorkloadSpec("topkshare", 2, 2 * group, 2, 128, dtype, 30000, 60000, "none", seed=119)
    w = W.make_workload(spec, DEV)
    W.make_dyadic_(w, seed=120)
    w.scale = 0.125
    n0, n1 = (int(x) for x in w.seq_lens)
    ranges = [(0, 0, n0 - 500), (1, 100, 9000), (1, 9000, n1)]
    for _ in range(2):
        _check_exact(w, ranges, [0, 1, 3], top_k, "%s G=%d k=%d span=%d" % (dtype, group, top_k, span))


@pytest.mark.parametrize("span", [0, 2048])
@pytest.mark.parametrize("order", ["ascending", "descending", "equal"])
def test_orders_that_defeat_the_bound(order, span):
    """Logits that rise with the token index pass every running bound (the scan writes all of
    them out), falling ones pass none after the start, equal ones all tie: the result is the same
    selection, with ties going to the earlier token."""
    hg.hg_attn_set_span_tokens(span)
    N, d, group = 20000, 128, 8
    spec = W.WorkloadSpec("topkorder", 1, group, 1, d, "f16", N, N, "none", seed=115)
    w = W.make_workload(spec, DEV)
    w.scale = 0.125
    w.q.zero_()
    w.q[..., 0] = 1.0
    w.k.zero_()
    steps = torch.arange(N, device=DEV) // 16  # 16 equal logits in a row: exact in fp16 up to 2048
    col = {"ascending": steps, "descending": (N // 16) - steps, "equal": torch.zeros_like(steps)}[order]
    w.k[0, 0, :, 0] = col.to(torch.float16)
    for top_k in (40, 128, 250):
        _check_exact(w, [(0, 0, 7000), (0, 7000, N)], [0, 2], top_k, "%s k=%d" % (order, top_k))


@pytest.mark.parametrize("group", [8, 1])
def test_long_and_short_survivor_lists_in_one_call(group):
    """One sequence whose logits rise with the token index (every logit passes the scan: a list
    too long for the one-workgroup selection) beside one with random logits (a short list): the
    selection behind the scan takes each (group, head) by the length of its own list."""
    N = 30000
    spec = W.WorkloadSpec("topkmixed", 2, group, 1, 128, "f16", N, N, "none", seed=131)
    w = W.make_workload(spec, DEV)
    W.make_dyadic_(w, seed=132)
    w.scale = 0.125
    w.q[0].zero_()
    w.q[0, :, 0] = 1.0
    w.k[0].zero_()
    w.k[0, 0, :, 0] = (torch.arange(N, device=DEV) // 16).to(torch.float16)  # exact in fp16 up to 2048
    for top_k in (50, 256):
        _check_exact(w, [(0, 0, N), (1, 0, 11000), (1, 11000, N)], [0, 1, 3], top_k, "G=%d k=%d" % (group, top_k))


@pytest.mark.parametrize("batch", [4, 5])
def test_more_slices_than_selection_workgroups(batch):
    """Many (group, head) pairs, so that the selection behind the scan launches two workgroups
    per pair (4 sequences x 64 heads) or one (5 sequences), and one sequence whose logits rise
    with the token index: its 40000 survivors per head are three slices, which the workgroups
    take in turn before the last one to finish selects among the candidates of all."""
    N, group, hkv = 40000, 8, 8
    spec = W.WorkloadSpec("topkslices", batch, group * hkv, hkv, 128, "f16", N, N, "none", seed=133)
    w = W.make_workload(spec, DEV)
    W.make_dyadic_(w, seed=134)
    w.scale = 0.125
    b = batch - 2
    w.q[b].zero_()
    w.q[b, :, 0] = 1.0
    w.k[b].zero_()
    w.k[b, :, :, 0] = (torch.arange(N, device=DEV) // 32).to(torch.float16)  # exact in fp16 up to 2048
    ranges = [(i, 0, N) for i in range(batch)]
    _check_exact(w, ranges, list(range(batch + 1)), 128, "B=%d" % batch)


@pytest.mark.parametrize("dtype,d,group", [("f16", 128, 8), ("bf16", 128, 4), ("f16", 128, 3), ("f16", 128, 1), ("f16", 64, 4)])
@pytest.mark.parametrize("top_k", [100, 256])
def test_equals_logits_then_select_and_is_valid_against_the_oracle(dtype, d, group, top_k):
    spec = W.WorkloadSpec("topkrnd", 2, 2 * group, 2, d, dtype, 9000, 40000, "none", outlier_k=True, seed=116 + group)
    w = W.make_workload(spec, DEV)
    rng = np.random.default_rng(117)
    ranges, gp = _groups_per_sequence(w, rng)
    sel, m, l, o = hg.hg_attn_topk(w.q, w.k, w.v, w.seq_lens, ranges, gp, top_k, w.scale)
    lg = hg.hg_attn_logits(w.q, w.k, w.v, w.seq_lens, ranges, w.scale)
    sel2, m2, l2, o2 = hg.hg_attn_select(w.q, w.k, w.v, w.seq_lens, ranges, lg, gp, top_k, w.scale)
    assert torch.equal(sel, sel2), "fused scan and logits -> select keep different tokens"
    assert torch.equal(m, m2)
    assert (l - l2).abs().max().item() <= 1e-4 * l2.abs().max().item() and (o - o2).abs().max().item() <= 1e-3
    # against the oracle: exact logits of every offloaded token
    qn, (kn, vn) = to_np(w.q), kv_np(w)
    exact = oracle.attn_logits(qn, kn, vn, w.seq_lens, w.scale, ranges)
    assert np.abs(to_np(lg).astype(np.float64) - exact).max() <= LOGIT_TOL
    pre = np.cumsum([0] + [e - s for _, s, e in ranges])
    got = to_np(sel)
    for g in range(len(gp) - 1):
        toks = np.concatenate([np.arange(s, e) for _, s, e in ranges[gp[g]:gp[g + 1]]] or [np.zeros(0, int)])
        for h in range(2 * group):
            row = exact[h, pre[gp[g]]:pre[gp[g + 1]]]
            kept = got[g, h][got[g, h] >= 0]
            keep = min(top_k, row.size)
            assert kept.size == keep and np.all(np.diff(kept) > 0) and np.isin(kept, toks).all()
            if keep == 0:
                continue
            kth = np.sort(row)[-keep]
            of_tok = dict(zip(toks.tolist(), row.tolist()))
            kept_vals = np.array([of_tok[t] for t in kept.tolist()])
            assert kept_vals.min() >= kth - 2 * LOGIT_TOL, "a kept token is clearly below the k-th largest logit"
            missing = np.setdiff1d(toks, kept)
            if missing.size:
                assert max(of_tok[t] for t in missing.tolist()) <= kth + 2 * LOGIT_TOL, "a clearly larger logit was dropped"
    gm, gl, go = oracle.attn_gather(qn, kn, vn, w.seq_lens, w.scale, list(range(len(gp) - 1)), got)
    check_triples(m, l, o, gm, gl, go, "triple over the kept list")


def test_long_group_takes_the_scan_by_itself_and_matches_the_two_call_sequence():
    """One 600k-token group, top_k 128: long enough for the library to choose the filtering scan;
    forced to the two-call sequence it must keep the same tokens."""
    spec = W.WorkloadSpec("topklong", 1, 8, 1, 128, "f16", 600000, 600000, "none", outlier_k=True, seed=121)
    w = W.make_workload(spec, DEV)
    ranges, gp = [(0, 0, 300000), (0, 300000, 590000)], [0, 2]
    hg.hg_attn_set_topk_mode(0)
    sel, m, l, o = hg.hg_attn_topk(w.q, w.k, w.v, w.seq_lens, ranges, gp, 128, w.scale)
    hg.hg_attn_set_topk_mode(2)
    sel2, m2, l2, o2 = hg.hg_attn_topk(w.q, w.k, w.v, w.seq_lens, ranges, gp, 128, w.scale)
    assert torch.equal(sel, sel2) and torch.equal(m, m2)
    assert (o - o2).abs().max().item() <= 1e-3
    gm, gl, go = oracle.attn_gather(to_np(w.q), *kv_np(w), w.seq_lens, w.scale, [0], to_np(sel))
    check_triples(m, l, o, gm, gl, go, "long group")


def test_full_cover_reproduces_unsplit_attention():
    """top_k at least as large as every group: nothing is dropped, and merged with the resident
    tokens the result is the unsplit attention."""
    spec = W.WorkloadSpec("topkall", 2, 8, 1, 128, "f16", 150, 240, "none", seed=118)
    w = W.make_workload(spec, DEV)
    off = [(b, 0, int(n) - 30) for b, n in enumerate(w.seq_lens)]
    res = [(b, int(n) - 30, int(n)) for b, n in enumerate(w.seq_lens)]
    _, m, l, o = hg.hg_attn_topk(w.q, w.k, w.v, w.seq_lens, off, [0, 1, 2], 256, w.scale)
    pm, pl, po = hg.hg_attn_partial(w.q, w.k, w.v, w.seq_lens, res, w.scale)
    out, lse = hg.hg_attn_merge2(m, l, o, [0, 1, 2], pm, pl, po, [0, 1, 2])
    ref, rlse = oracle.attn_full(to_np(w.q), *kv_np(w), w.seq_lens, w.scale)
    check_out(out, lse, ref, rlse, "top_k covers the offloaded tokens")

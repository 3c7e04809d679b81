"""GPU parity of hg_attn_gather: attention statistics over a LISTED token set per (group, query
head) -- the executor's side of a selection decided elsewhere (Pre-QK^T selection, or a Post-QK^T
list taken with a proxy query and evaluated with the true one).  Which rows are read is index work
and is pinned by exact integer sums; the triples match the oracle to the floating-point bars."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_18529_amd as hg
from paper_2604_18529_amd import workloads as W

from parity_utils import check_out, check_triples, kv_np, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _lists(seed, group_seq, seq_lens, hq, max_k, pad_frac=0.25, distinct=False):
    """Seeded token lists [G, Hq, max_k]: random positions of the group's sequence (duplicates
    allowed unless `distinct`), a share of entries replaced by negative padding."""
    rng = np.random.RandomState(seed)
    G = len(group_seq)
    idx = np.full((G, hq, max_k), -1, dtype=np.int32)
    for g, b in enumerate(group_seq):
        n = int(seq_lens[b])
        if n == 0:
            continue
        for h in range(hq):
            if distinct:
                row = rng.permutation(n)[:max_k].astype(np.int32)
                row = np.concatenate([row, np.full(max_k - row.size, -1, np.int32)])
            else:
                row = rng.randint(0, n, size=max_k).astype(np.int32)
            row[rng.random_sample(max_k) < pad_frac] = -1 - rng.randint(0, 7)
            idx[g, h] = row
    return idx


def _check_gather(w, group_seq, idx_np, what, **kw):
    idx = torch.from_numpy(idx_np).to(DEV)
    m, l, o = hg.hg_attn_gather(w.q, kw.pop("k", w.k), kw.pop("v", w.v), w.seq_lens, group_seq, idx, w.scale, **kw)
    rm, rl, ro = oracle.attn_gather(to_np(w.q), *kv_np(w), w.seq_lens, w.scale, group_seq, idx_np)
    check_triples(m, l, o, rm, rl, ro, what)
    torch.cuda.synchronize()
    return m, l, o


@pytest.mark.parametrize("max_k", [1, 3, 64, 129, 1000])
@pytest.mark.parametrize("dtype,d,group", [("f16", 128, 1), ("f16", 128, 8), ("f32", 64, 1), ("f16", 64, 2), ("f32", 128, 3),
                                            ("bf16", 128, 4), ("bf16", 64, 1)])
def test_every_storage_type_and_list_length(dtype, d, group, max_k):
    spec = W.WorkloadSpec("gather", 3, 2 * group, 2, d, dtype, 50, 2500, "none", seed=90 + group)
    w = W.make_workload(spec, DEV)
    group_seq = [2, 0, 0, 1, 2]  # several lists per sequence, in any order
    idx = _lists(91 + max_k, group_seq, w.seq_lens, 2 * group, max_k)
    idx[1, 0] = -1  # one list without tokens: (-inf, 0, 0)
    _check_gather(w, group_seq, idx, "%s d=%d G=%d k=%d" % (dtype, d, group, max_k))


@pytest.mark.parametrize("dtype,d", [("f16", 128), ("f32", 64), ("bf16", 64)])
def test_zero_query_counts_listings_and_bitplanes_exactly(dtype, d):
    """q = 0 and V[t][c] = bit c of t: l is the number of listings and O the per-bit counts over
    the listed tokens -- exact integers, so every listed row (and no other) was read, from the
    right sequence and KV head, duplicates as often as listed."""
    N = 40000
    spec = W.WorkloadSpec("gatherbits", 2, 4, 2, d, dtype, N, N, "none", seed=92)
    w = W.make_workload(spec, DEV)
    w.q.zero_()
    tdt = {"f16": torch.float16, "f32": torch.float32, "bf16": torch.bfloat16}[dtype]
    w.v[:, :] = W.bitplane_values(N, d, tdt, DEV)
    w.v[1, 1] = 0  # a different KV head / sequence would change the counts
    group_seq = [0, 1, 1]
    idx = _lists(93, group_seq, w.seq_lens, 4, 777)
    idx[0, 0, :4] = [0, N - 1, N - 1, 16383]
    m, l, o = hg.hg_attn_gather(w.q, w.k, w.v, w.seq_lens, group_seq, torch.from_numpy(idx).to(DEV), w.scale)
    rm, rl, ro = oracle.attn_gather(to_np(w.q), *kv_np(w), w.seq_lens, w.scale, group_seq, idx)
    assert np.array_equal(to_np(m).astype(np.float64), rm)
    assert np.array_equal(to_np(l).astype(np.float64), rl)
    assert np.array_equal(to_np(o).astype(np.float64), ro)
    assert rl[0, 0] == (idx[0, 0] >= 0).sum() and not ro[1:, 2:].any()


def test_whole_range_listed_equals_partial_and_merges_to_full():
    """Listing every token of [begin, end) in shuffled order gives that range's triple; merged
    with the triple of the remaining tokens it is the unsplit result."""
    spec = W.WorkloadSpec("gatherrange", 2, 8, 2, 128, "f16", 3000, 3000, "none", seed=94)
    w = W.make_workload(spec, DEV)
    rng = np.random.RandomState(95)
    idx = np.stack([np.stack([rng.permutation(np.arange(500, 2500)) for _ in range(8)]) for _ in range(2)]).astype(np.int32)
    m, l, o = _check_gather(w, [0, 1], idx, "range as list")
    pm, pl, po = hg.hg_attn_partial(w.q, w.k, w.v, w.seq_lens, [(0, 0, 500), (0, 2500, 3000), (1, 0, 500), (1, 2500, 3000)], w.scale)
    out, lse = hg.hg_attn_merge2(m, l, o, [0, 1, 2], pm, pl, po, [0, 2, 4])
    ref, rlse = oracle.attn_full(to_np(w.q), *kv_np(w), w.seq_lens, w.scale)
    check_out(out, lse, ref, rlse, "listed + resident merged")


@pytest.mark.parametrize("block_tokens", [16, 256])
@pytest.mark.parametrize("dtype,d,group", [("f16", 128, 4), ("f32", 64, 1), ("bf16", 64, 2)])
def test_paged_cache(dtype, d, group, block_tokens):
    spec = W.WorkloadSpec("gatherpaged", 3, 2 * group, 2, d, dtype, 1, 3000, "none", seed=96)
    w = W.make_workload(spec, DEV)
    kp, vp, table = W.make_paged(w, block_tokens, seed=7)
    group_seq = [0, 1, 2, 2]
    idx = _lists(97, group_seq, w.seq_lens, 2 * group, 200)
    _check_gather(w, group_seq, idx, "paged bt=%d" % block_tokens, k=kp, v=vp, block_table=table)


def test_token_major_layout():
    spec = W.WorkloadSpec("gathertm", 2, 4, 2, 128, "f16", 400, 900, "none", seed=98)
    w = W.make_workload(spec, DEV, layout="bthd")
    idx = _lists(99, [1, 0], w.seq_lens, 4, 100)
    _check_gather(w, [1, 0], idx, "token-major")


def test_many_groups_use_the_uploaded_table():
    """More groups than the kernel arguments carry: the sequence table travels through the
    workspace."""
    spec = W.WorkloadSpec("gathermany", 4, 2, 2, 64, "f16", 100, 300, "none", seed=100)
    w = W.make_workload(spec, DEV)
    rng = np.random.RandomState(101)
    group_seq = rng.randint(0, 4, size=700).tolist()
    idx = _lists(102, group_seq, w.seq_lens, 2, 9)
    _check_gather(w, group_seq, idx, "700 groups")


def test_proxy_selection_evaluated_with_the_true_query():
    """The flow the call exists for: the tokens are chosen with a proxy query (logits -> top-k),
    then the executor evaluates exactly those tokens with the true query.  The kept sets are
    bit-exact against the oracle's selection on the same fp32 logits; the gathered triples match
    the oracle's listed-token routine; merged with the resident tokens the result approaches the
    unsplit one as the list grows and equals it when the list covers the offloaded tokens."""
    spec = W.WorkloadSpec("gatherproxy", 2, 8, 2, 128, "f16", 4000, 6000, "none", seed=103)
    w = W.make_workload(spec, DEV)
    w.seq_lens[:] = [6000, 4000]
    cut = [4800, 3200]
    off = [(0, 0, cut[0]), (1, 0, cut[1])]
    res = [(0, cut[0], 6000), (1, cut[1], 4000)]
    qp = W.proxy_query(w.q, 0.95, seed=104)
    lg = hg.hg_attn_logits(qp, w.k, w.v, w.seq_lens, off, w.scale)
    qn, (kn, vn) = to_np(w.q), kv_np(w)
    ref, rlse = oracle.attn_full(qn, kn, vn, w.seq_lens, w.scale)
    rm_, rl_, ro_ = hg.hg_attn_partial(w.q, w.k, w.v, w.seq_lens, res, w.scale)
    errs = []
    for top_k in (64, 1024, 4096):
        sel, _, _, _ = hg.hg_attn_select(qp, w.k, w.v, w.seq_lens, off, lg, [0, 1, 2], top_k, w.scale)
        rsel, _, _, _ = oracle.attn_select(to_np(qp), kn, vn, w.seq_lens, w.scale, off, to_np(lg), [0, 1, 2], top_k)
        assert np.array_equal(to_np(sel), rsel)
        m, l, o = hg.hg_attn_gather(w.q, w.k, w.v, w.seq_lens, [0, 1], sel, w.scale)
        gm, gl, go = oracle.attn_gather(qn, kn, vn, w.seq_lens, w.scale, [0, 1], rsel)
        check_triples(m, l, o, gm, gl, go, "gather of proxy top-%d" % top_k)
        out, lse = hg.hg_attn_merge2(m, l, o, [0, 1, 2], rm_, rl_, ro_, [0, 1, 2])
        errs.append(np.abs(to_np(out).astype(np.float64) - ref).max())
    assert errs[0] > errs[1] > errs[2] or errs[1] < 2e-3
    # sequence 1's 3200 offloaded tokens are all inside the 4096 kept: exact there
    assert np.abs(to_np(out[1]).astype(np.float64) - ref[1]).max() <= 2e-3
    assert np.abs(to_np(lse[1]).astype(np.float64) - rlse[1]).max() <= 1e-3


def test_rejects_bad_arguments():
    spec = W.WorkloadSpec("gatherrej", 2, 2, 2, 64, "f16", 100, 100, "none", seed=105)
    w = W.make_workload(spec, DEV)
    idx = torch.zeros((1, 2, 4), dtype=torch.int32, device=DEV)
    with pytest.raises(hg.HgError) as ei:
        hg.hg_attn_gather(w.q, w.k, w.v, w.seq_lens, [2], idx, w.scale)
    assert ei.value.status == -4
    with pytest.raises(ValueError):
        hg.hg_attn_gather(w.q, w.k, w.v, w.seq_lens, [0], idx.to(torch.int64), w.scale)

"""GPU parity of Post-QK^T selection (hg_attn_select): which tokens are kept is integer work and
must match the oracle bit for bit when both decide on the same fp32 logits; the folded triple
matches to the floating-point bars."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_18529_amd as hg
from paper_2604_18529_amd import workloads as W

from parity_utils import check_out, check_triples, kv_np, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _seeded_logits(hq, ltok, seed, ties):
    """fp32 logits as an INPUT (seeded, not produced by either side).  `ties` quantises them so
    that many values collide exactly and the tie-break is exercised."""
    rng = np.random.RandomState(seed)
    lg = (rng.standard_normal((hq, ltok)) * 3).astype(np.float32)
    if ties:
        lg = (np.round(lg * 8) / 8).astype(np.float32)
    return lg


def _check_select(w, ranges, gp, lg_np, top_k, what):
    lg = torch.from_numpy(lg_np).to(DEV)
    sel, m, l, o = hg.hg_attn_select(w.q, w.k, w.v, w.seq_lens, ranges, lg, gp, top_k, w.scale)
    rsel, rm, rl, ro = oracle.attn_select(to_np(w.q), *kv_np(w), w.seq_lens, w.scale, ranges, lg_np, gp, top_k)
    assert np.array_equal(to_np(sel), rsel), what + ": kept tokens differ"
    m_g = to_np(m).astype(np.float64)
    fin = np.isfinite(rm)
    assert np.array_equal(m_g[fin], rm[fin]), what + ": m must be the kept maximum exactly"
    check_triples(m, l, o, rm, rl, ro, what)
    return sel, m, l, o


@pytest.mark.parametrize("ties", [False, True])
@pytest.mark.parametrize("top_k", [1, 7, 128, 1000, 4096])
def test_selection_is_bit_exact_on_given_logits(top_k, ties):
    spec = W.WorkloadSpec("sel", 3, 4, 2, 128, "f16", 100, 6000, "none", seed=51)
    w = W.make_workload(spec, DEV)
    w.seq_lens[:] = [6000, 100, 2500]
    ranges = [(0, 0, 2500), (0, 2500, 2500), (0, 3000, 6000), (1, 0, 100), (2, 10, 2500)]
    gp = [0, 3, 4, 5]
    ltok = sum(e - s for _, s, e in ranges)
    _check_select(w, ranges, gp, _seeded_logits(4, ltok, 52 + top_k, ties), top_k, "k=%d ties=%s" % (top_k, ties))


@pytest.mark.parametrize("dtype,d,group", [("f16", 128, 8), ("f32", 64, 1), ("f16", 64, 2), ("f32", 128, 3)])
def test_every_storage_type(dtype, d, group):
    spec = W.WorkloadSpec("selinst", 2, 2 * group, 2, d, dtype, 300, 900, "ratios", 2, seed=53)
    w = W.make_workload(spec, DEV)
    ltok = sum(e - s for _, s, e in w.ranges)
    _check_select(w, w.ranges, w.group_ptr, _seeded_logits(2 * group, ltok, 54, True), 50, "%s d=%d G=%d" % (dtype, d, group))


def test_edge_groups():
    """An empty group, a group of empty ranges, a one-token group, all-equal logits (the first
    top_k columns win), and more ranges/groups than fit in kernel arguments."""
    spec = W.WorkloadSpec("seledge", 3, 2, 2, 128, "f16", 0, 500, "none", seed=55)
    w = W.make_workload(spec, DEV)
    w.seq_lens[:] = [500, 0, 1]
    ranges = [(0, 0, 0), (0, 7, 7), (2, 0, 1), (0, 0, 500)]
    gp = [0, 2, 2, 3, 4]
    lg = _seeded_logits(2, 501, 56, True)
    lg[:, 1:] = 2.5  # group 3: every logit equal
    sel, m, l, o = _check_select(w, ranges, gp, lg, 16, "edge")
    assert to_np(sel[3, 0]).tolist() == list(range(16))
    assert np.all(to_np(sel[0]) == -1) and np.all(to_np(sel[1]) == -1)
    spec = W.WorkloadSpec("selmany", 2, 4, 4, 64, "f16", 3000, 3000, "none", seed=57)
    w = W.make_workload(spec, DEV)
    ranges, gp = [], [0]
    for b in range(2):
        for i in range(300):
            ranges.append((b, 10 * i, 10 * i + 9))
            gp.append(len(ranges))
    _check_select(w, ranges, gp, _seeded_logits(4, 2 * 300 * 9, 58, False), 4, "many")


def test_post_qk_selection_end_to_end():
    """The whole Post-QK^T flow on the GPU: logits of the offloaded (old) tokens, top-k, triple,
    merge with the resident (recent) tokens' triple.  The oracle runs the same flow on its own
    logits; kept sets may differ only where logits are within rounding of the threshold, and the
    merged outputs agree to the output bar.  With top_k >= the offloaded count the flow is exact
    attention."""
    spec = W.WorkloadSpec("postqk", 2, 8, 2, 128, "f16", 3000, 5000, "none", seed=59)
    w = W.make_workload(spec, DEV)
    old = [(b, 0, int(0.8 * n)) for b, n in enumerate(w.seq_lens)]
    new = [(b, int(0.8 * n), int(n)) for b, n in enumerate(w.seq_lens)]
    gp_old = np.arange(spec.batch + 1, dtype=np.int32)
    qn = to_np(w.q)
    kn, vn = kv_np(w)
    lg_ref = oracle.attn_logits(qn, kn, vn, w.seq_lens, w.scale, old)
    pm, pl, po = oracle.attn_partial(qn, kn, vn, w.seq_lens, w.scale, new)
    m2, l2, o2 = hg.hg_attn_partial(w.q, w.k, w.v, w.seq_lens, new, w.scale)
    lg = hg.hg_attn_logits(w.q, w.k, w.v, w.seq_lens, old, w.scale)
    merge_gp = np.arange(0, 2 * spec.batch + 1, 2, dtype=np.int32)
    idx = torch.arange(2 * spec.batch, device=DEV).reshape(2, spec.batch).t().reshape(-1)
    idn = np.arange(2 * spec.batch).reshape(2, spec.batch).T.reshape(-1)
    for top_k in (128, 4096):
        sel, m1, l1, o1 = hg.hg_attn_select(w.q, w.k, w.v, w.seq_lens, old, lg, gp_old, top_k, w.scale)
        out, lse = hg.hg_attn_merge(torch.cat([m1, m2])[idx].contiguous(), torch.cat([l1, l2])[idx].contiguous(),
                                    torch.cat([o1, o2])[idx].contiguous(), merge_gp)
        rsel, rm, rl, ro = oracle.attn_select(qn, kn, vn, w.seq_lens, w.scale, old, lg_ref.astype(np.float32), gp_old, top_k)
        ref, rlse = oracle.attn_merge(np.concatenate([rm, pm])[idn], np.concatenate([rl, pl])[idn],
                                      np.concatenate([ro, po])[idn], merge_gp)
        check_out(out, lse, ref, rlse, "post-qk k=%d" % top_k)
        # kept sets: identical except for tokens whose logit is within rounding of the threshold
        sel_np = to_np(sel)
        col0 = 0
        for b in range(spec.batch):
            n_old = old[b][2]
            for h in range(spec.n_q_heads):
                got, want = set(sel_np[b, h][sel_np[b, h] >= 0].tolist()), set(rsel[b, h][rsel[b, h] >= 0].tolist())
                assert len(got) == len(want) == min(top_k, n_old)
                row = lg_ref[h, col0:col0 + n_old]
                thr = np.sort(row)[-min(top_k, n_old)]
                for t in got ^ want:
                    assert abs(row[t] - thr) <= 1e-4
            col0 += n_old
        if top_k >= max(r[2] for r in old):
            exact, elsE = oracle.attn_full(qn, kn, vn, w.seq_lens, w.scale)
            check_out(out, lse, exact, elsE, "post-qk keeps everything")


@pytest.mark.parametrize("top_k", [5, 4096])
def test_long_groups_take_the_two_stage_path(top_k):
    """Groups longer than 16384 tokens are cut into parts whose candidates are merged; the kept
    set must still be the exact global top-k with the global tie-break (lower column)."""
    spec = W.WorkloadSpec("sellong", 2, 2, 1, 128, "f16", 70000, 150000, "none", seed=62)
    w = W.make_workload(spec, DEV)
    w.seq_lens[:] = [150000, 70000]
    ranges = [(0, 0, 90000), (0, 90000, 150000), (1, 100, 70000)]
    gp = [0, 2, 3]
    ltok = sum(e - s for _, s, e in ranges)
    lg = _seeded_logits(2, ltok, 63, True)
    lg[1, :] = 1.25  # one head with every logit equal: the first top_k columns of each group win
    sel, _, _, _ = _check_select(w, ranges, gp, lg, top_k, "two-stage k=%d" % top_k)
    assert to_np(sel[0, 1]).tolist() == list(range(top_k))
    assert to_np(sel[1, 1]).tolist() == list(range(100, 100 + top_k))


@pytest.mark.parametrize("order", ["ascending", "descending", "sawtooth", "two_values"])
@pytest.mark.parametrize("n", [1000, 16384, 40000])
def test_adversarial_orders(order, n):
    """Orders that defeat the lower bound taken from per-thread maxima (every large logit in the
    same few threads, or in the last columns), and logits with two distinct values only."""
    spec = W.WorkloadSpec("seladv", 1, 2, 1, 64, "f16", n, n, "none", seed=64)
    w = W.make_workload(spec, DEV)
    ranges, gp = [(0, 0, n)], [0, 1]
    base = np.arange(n, dtype=np.float32) / 64
    if order == "ascending":
        rows = [base, base * 0.5]
    elif order == "descending":
        rows = [base[::-1], -base]
    elif order == "sawtooth":
        rows = [(np.arange(n) % 1024).astype(np.float32), (np.arange(n) % 1024 == 3).astype(np.float32) * 5]
    else:
        rng = np.random.default_rng(65)
        rows = [(rng.random(n) < 0.01).astype(np.float32), (rng.random(n) < 0.9).astype(np.float32) - 2]
    lg = np.ascontiguousarray(np.stack(rows).astype(np.float32))
    for top_k in (3, 128, 256, 1000, 2000):
        _check_select(w, ranges, gp, lg, top_k, "%s n=%d k=%d" % (order, n, top_k))


@pytest.mark.parametrize("n,finite", [(20000, 14000), (1000, 50), (40000, 100)])
def test_masked_logits(n, finite):
    """Logits of masked tokens are -inf.  With fewer finite logits than top_k the kept set is the
    finite ones plus the first masked columns, whose weights are exactly zero."""
    spec = W.WorkloadSpec("selmask", 1, 2, 1, 64, "f16", n, n, "none", seed=68)
    w = W.make_workload(spec, DEV)
    ranges, gp = [(0, 0, n)], [0, 1]
    rng = np.random.default_rng(69)
    lg = np.full((2, n), -np.inf, dtype=np.float32)
    for h in range(2):
        cols = rng.choice(n, size=finite, replace=False)
        lg[h, cols] = rng.standard_normal(finite).astype(np.float32)
    _check_select(w, ranges, gp, lg, 128, "masked n=%d finite=%d" % (n, finite))


def test_middle_stage_and_pads_below_masked_logits():
    """19 parts x top_k 1000 candidates are more than one workgroup takes at once: a middle stage
    reduces them first.  The second group is tiny and mostly masked: all its tokens are kept, the
    -inf ones included, although its parts are nearly all padding."""
    n0, n1 = 300_000, 50
    spec = W.WorkloadSpec("selmid", 2, 2, 1, 64, "f16", n1, n0, "none", seed=76)
    w = W.make_workload(spec, DEV)
    w.seq_lens[:] = [n0, n1]
    ranges, gp = [(0, 0, 200_000), (0, 200_000, n0), (1, 0, n1)], [0, 2, 3]
    rng = np.random.default_rng(77)
    lg = (np.round(rng.standard_normal((2, n0 + n1)) * 16) / 16).astype(np.float32)
    lg[:, n0:] = -np.inf
    lg[:, n0 + rng.choice(n1, 10, replace=False)] = 0.5
    lg[1, :n0] = np.sort(lg[1, :n0])  # sorted row: every kept token in the last parts
    sel, _, _, _ = _check_select(w, ranges, gp, lg, 1000, "middle stage")
    assert to_np(sel[1, 0][:n1]).tolist() == list(range(n1))


def test_signed_zeros_tie():
    """-0.0 and +0.0 are the same logit: at a threshold of zero the lower column wins whatever the
    sign bits say."""
    n = 600
    spec = W.WorkloadSpec("selzero", 1, 2, 1, 64, "f16", n, n, "none", seed=74)
    w = W.make_workload(spec, DEV)
    rng = np.random.default_rng(75)
    lg = np.where(rng.random((2, n)) < 0.5, np.float32(-0.0), np.float32(0.0)).astype(np.float32)
    lg[0, rng.choice(n, 20, replace=False)] = 1.0
    lg[1, rng.choice(n, 300, replace=False)] = -1.0
    for top_k in (50, 200, 1000):
        sel, _, _, _ = _check_select(w, [(0, 0, n)], [0, 1], lg, top_k, "signed zeros k=%d" % top_k)
    sel, _, _, _ = _check_select(w, [(0, 0, n)], [0, 1], lg, 50, "signed zeros")
    ones = np.flatnonzero(lg[0] == 1.0)
    zeros = np.flatnonzero(lg[0] == 0.0)[:30]
    assert to_np(sel[0, 0]).tolist() == sorted(ones.tolist() + zeros.tolist())


def test_groups_beyond_the_part_limit():
    """A group of more than 64 x 16384 tokens leaves parts that do not fit in registers: the
    streaming variant of the candidates stage runs.  Sorted logits put every kept token in the last part."""
    n = 1_200_000
    spec = W.WorkloadSpec("selhuge", 1, 1, 1, 64, "f16", n, n, "none", seed=66)
    w = W.make_workload(spec, DEV)
    ranges, gp = [(0, 0, 500_000), (0, 500_000, n)], [0, 2]
    rng = np.random.default_rng(67)
    lg = np.sort(rng.standard_normal(n).astype(np.float32))[None, :]
    lg = np.ascontiguousarray(np.round(lg * 256) / 256)
    sel, _, _, _ = _check_select(w, ranges, gp, lg, 500, "huge group")
    assert int(to_np(sel[0, 0]).min()) > n - 40000


def test_bad_arguments():
    spec = W.WorkloadSpec("selerr", 1, 2, 2, 64, "f16", 100, 100, "none", seed=60)
    w = W.make_workload(spec, DEV)
    lg = torch.zeros((2, 100), dtype=torch.float32, device=DEV)
    for k in (0, 4097):
        with pytest.raises(hg.HgError) as ei:
            hg.hg_attn_select(w.q, w.k, w.v, w.seq_lens, w.ranges, lg, [0, 1], k, w.scale)
        assert ei.value.status == -2


@pytest.mark.parametrize("top_k", [128, 1024, 2048])
def test_full_size_million_token_group(top_k):
    """Benchmark shape: 64 query heads over 8 KV heads, one group of 1,048,576 offloaded tokens;
    sampled heads against the oracle on seeded logits.  top_k = 128: fast path in both stages;
    1024: fast first stage, radix passes over the 64 x 1024 candidates; 2048: radix passes in both."""
    spec = W.WORKLOADS[4]
    w = W.make_workload(spec, DEV)
    n = int(w.seq_lens[0])
    gen = torch.Generator(device=DEV)
    gen.manual_seed(61)
    lg = (torch.randn((spec.n_q_heads, n), generator=gen, device=DEV, dtype=torch.float32) * 2)
    lg = (lg * 64).round() / 64  # exact ties
    ranges, gp = [(0, 0, n)], [0, 1]
    sel, m, l, o = hg.hg_attn_select(w.q, w.k, w.v, w.seq_lens, ranges, lg, gp, top_k, w.scale)
    G = spec.n_q_heads // spec.n_kv_heads
    for h in (0, 13, 63):
        qs = to_np(w.q[:, h:h + 1])
        ks = to_np(w.k[:, h // G:h // G + 1])
        vs = to_np(w.v[:, h // G:h // G + 1])
        rsel, rm, rl, ro = oracle.attn_select(qs, ks, vs, [n], w.scale, ranges, to_np(lg[h:h + 1]), gp, top_k)
        assert np.array_equal(to_np(sel[0, h]), rsel[0, 0])
        check_triples(m[:, h:h + 1], l[:, h:h + 1], o[:, h:h + 1], rm, rl, ro, "1M head %d" % h)

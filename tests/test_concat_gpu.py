"""GPU parity of the paper-literal route: hg_attn_logits (raw logits per range, the paper's wire
format) and hg_attn_concat (one softmax over a group's concatenated logits, then P.V), against the
oracle's attn_logits / attn_concat on the same bits."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_18529_amd as hg
from paper_2604_18529_amd import workloads as W

from parity_utils import LSE_TOL, OUT_TOL, check_out, kv_np, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
LOGIT_TOL = 1e-3


@pytest.fixture(autouse=True)
def _default_spans():
    hg.hg_attn_set_span_tokens(0)
    yield
    hg.hg_attn_set_span_tokens(0)


def _oracle_concat(w, ranges, group_ptr):
    """Oracle output per GROUP: attn_concat works per sequence, so each group is run on its own."""
    qn = to_np(w.q)
    kn, vn = kv_np(w)
    outs, lses = [], []
    for i in range(len(group_ptr) - 1):
        rs = ranges[group_ptr[i]:group_ptr[i + 1]]
        if not rs or all(e == s for _, s, e in rs):
            outs.append(np.zeros((w.q.shape[1], w.q.shape[2])))
            lses.append(np.full(w.q.shape[1], -np.inf))
            continue
        b = rs[0][0]
        full = oracle.attn_concat(qn, kn, vn, w.seq_lens, w.scale, rs)
        lg = oracle.attn_logits(qn, kn, vn, w.seq_lens, w.scale, rs)
        outs.append(full[b])
        mx = lg.max(axis=1)
        lses.append(mx + np.log(np.exp(lg - mx[:, None]).sum(axis=1)))
    return np.stack(outs), np.stack(lses)


def _check_logits(w, ranges, lg):
    ref = oracle.attn_logits(to_np(w.q), *kv_np(w), w.seq_lens, w.scale, ranges)
    got = to_np(lg).astype(np.float64)
    assert got.shape == ref.shape
    if ref.size:
        assert np.abs(got - ref).max() <= LOGIT_TOL
    return ref


def _run(w, ranges=None, group_ptr=None, what=""):
    ranges = w.ranges if ranges is None else ranges
    group_ptr = w.group_ptr if group_ptr is None else group_ptr
    lg = hg.hg_attn_logits(w.q, w.k, w.v, w.seq_lens, ranges, w.scale)
    _check_logits(w, ranges, lg)
    out, lse = hg.hg_attn_concat(w.q, w.k, w.v, w.seq_lens, ranges, lg, group_ptr, w.scale)
    ref, rlse = _oracle_concat(w, ranges, group_ptr)
    check_out(out, lse, ref, rlse, what + " concat")
    return lg, out, lse


def test_config0_tiny():
    w = W.make_workload(W.WORKLOADS[0], DEV)
    _run(w, what="config0")


REDUCED = [
    W.WORKLOADS[1].scaled(name="r1", batch=2, n_q_heads=8, n_kv_heads=8, n_min=3000, n_max=3000),
    W.WORKLOADS[2].scaled(name="r2", batch=4, n_q_heads=5, n_kv_heads=5, n_min=1500, n_max=3100),
    W.WORKLOADS[3].scaled(name="r3", batch=2, n_q_heads=7, n_kv_heads=7, n_min=5000, n_max=5000),
    W.WORKLOADS[4].scaled(name="r4", batch=1, n_q_heads=16, n_kv_heads=2, n_min=9001, n_max=9001),
]


@pytest.mark.parametrize("spec", REDUCED, ids=lambda s: s.name)
@pytest.mark.parametrize("span", [0, 64, 1024])
def test_reduced_configs(spec, span):
    hg.hg_attn_set_span_tokens(span)
    w = W.make_workload(spec, DEV)
    _run(w, what="%s span=%d" % (spec.name, span))


@pytest.mark.parametrize("dtype", ["f16", "f32"])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("group", [1, 2, 3, 4, 5, 8, 16])
def test_every_kernel_instance(dtype, d, group):
    spec = W.WorkloadSpec("inst", 3, 2 * group, 2, d, dtype, 1, 700, "ratios", 3, seed=group + d)
    w = W.make_workload(spec, DEV)
    _run(w, what="%s d=%d G=%d" % (dtype, d, group))


@pytest.mark.parametrize("dtype,d,hq,hkv", [("f16", 128, 3, 3), ("f16", 64, 2, 2), ("f32", 128, 8, 2), ("f16", 128, 16, 2), ("bf16", 128, 6, 1)],
                         ids=["mha-f16-d128", "mha-f16-d64", "vector-kernel-4-heads", "matrix-core-8-heads", "matrix-core-6-heads-bf16"])
@pytest.mark.parametrize("span", [0, 64, 50048])
def test_logits_window_long_streams_many_ranges(dtype, d, hq, hkv, span):
    """The logits are collected in an LDS window that is written out when full and runs on across
    range boundaries: streams far longer than the window (32768 logits per head chunk in the vector
    kernel, fewer with several heads; 1472-12160 tokens in the matrix-core kernel), cut into many
    ragged ranges, under spans that start windows in the middle of a stream.  The output starts as
    NaN, so a column that is never written, or written from a stale window, shows."""
    spec = W.WorkloadSpec("window", 2, hq, hkv, d, dtype, 70000, 90000, "dirichlet", 23, seed=77 + hq + d)
    w = W.make_workload(spec, DEV)
    for ranges in (w.ranges, [r for i, r in enumerate(w.ranges) if i % 5 != 2][::-1]):  # tiling; with gaps, in reverse order
        hg.hg_attn_set_span_tokens(span)
        ltok = sum(e - b for (_, b, e) in ranges)
        lg = torch.full((hq, ltok), float("nan"), dtype=torch.float32, device=DEV)
        hg.hg_attn_logits(w.q, w.k, w.v, w.seq_lens, ranges, w.scale, logits=lg)
        torch.cuda.synchronize()
        assert not torch.isnan(lg).any()
        _check_logits(w, ranges, lg)


def test_concat_equals_statistics_route():
    """The paper's concatenate-then-softmax and the (m, l, O) merge are the same function."""
    spec = W.WorkloadSpec("same", 2, 8, 2, 128, "f16", 3000, 4000, "dirichlet", 6, seed=31)
    w = W.make_workload(spec, DEV)
    _, out, lse = _run(w, what="same")
    m, l, o = hg.hg_attn_partial(w.q, w.k, w.v, w.seq_lens, w.ranges, w.scale)
    mout, mlse = hg.hg_attn_merge(m, l, o, w.group_ptr)
    assert (out - mout).abs().max().item() <= 2e-5
    assert (lse - mlse).abs().max().item() <= 2e-5


def test_logits_from_another_executor():
    """Hybrid execution as the paper describes it: the logits of the OLD half of every cache come
    from the CPU (here: the oracle's logits, rounded to fp32), those of the recent half from the
    GPU; the GPU concatenates, applies one softmax and aggregates V."""
    spec = W.WorkloadSpec("hybrid", 2, 4, 4, 128, "f16", 2500, 2500, "half", 2, seed=32)
    w = W.make_workload(spec, DEV)
    cpu_ranges = [r for i, r in enumerate(w.ranges) if i % 2 == 0]  # tokens [0, N/2) of each sequence
    gpu_ranges = [r for i, r in enumerate(w.ranges) if i % 2 == 1]
    cpu_lg = oracle.attn_logits(to_np(w.q), *kv_np(w), w.seq_lens, w.scale, cpu_ranges).astype(np.float32)
    gpu_lg = hg.hg_attn_logits(w.q, w.k, w.v, w.seq_lens, gpu_ranges, w.scale)
    # concatenate in the order of the full table: per sequence, CPU part then GPU part
    cols, c_off, g_off = [], 0, 0
    cpu_t = torch.from_numpy(cpu_lg).to(DEV)
    for i, (_, s, e) in enumerate(w.ranges):
        n = e - s
        if i % 2 == 0:
            cols.append(cpu_t[:, c_off:c_off + n]); c_off += n
        else:
            cols.append(gpu_lg[:, g_off:g_off + n]); g_off += n
    lg = torch.cat(cols, dim=1).contiguous()
    out, lse = hg.hg_attn_concat(w.q, w.k, w.v, w.seq_lens, w.ranges, lg, w.group_ptr, w.scale)
    ref, rlse = oracle.attn_full(to_np(w.q), *kv_np(w), w.seq_lens, w.scale)
    check_out(out, lse, ref, rlse, "hybrid")


def test_edge_tables():
    """Empty ranges, an empty group, a group of only empty ranges, one-token ranges, unordered
    ranges inside a group, more ranges and groups than fit in kernel arguments."""
    hg.hg_attn_set_span_tokens(64)
    spec = W.WorkloadSpec("edge", 3, 4, 2, 128, "f16", 0, 1000, "none", seed=33)
    w = W.make_workload(spec, DEV)
    w.seq_lens[:] = [1000, 0, 257]
    ranges = [(0, 500, 1000), (0, 0, 0), (0, 0, 500), (1, 0, 0), (2, 0, 1), (2, 1, 257), (2, 100, 100)]
    gp = [0, 3, 3, 4, 7]
    _run(w, ranges, gp, "edge")
    out, lse = hg.hg_attn_concat(w.q, w.k, w.v, w.seq_lens, ranges,
                                 hg.hg_attn_logits(w.q, w.k, w.v, w.seq_lens, ranges, w.scale), gp, w.scale)
    assert not to_np(out[1]).any() and np.isneginf(to_np(lse[1])).all()
    assert not to_np(out[2]).any() and np.isneginf(to_np(lse[2])).all()
    # many ranges / many groups
    spec = W.WorkloadSpec("many", 2, 4, 4, 64, "f16", 2000, 2000, "none", seed=34)
    w = W.make_workload(spec, DEV)
    ranges, gp = [], [0]
    for b in range(2):
        for i in range(200):
            ranges.append((b, 10 * i, 10 * i + 7))
            if i % 1 == 0:
                gp.append(len(ranges))
    _run(w, ranges, gp, "many")


def test_bad_groups_are_rejected():
    spec = W.WorkloadSpec("err", 2, 2, 2, 64, "f16", 100, 100, "half", 2, seed=35)
    w = W.make_workload(spec, DEV)
    lg = hg.hg_attn_logits(w.q, w.k, w.v, w.seq_lens, w.ranges, w.scale)
    for bad in ([0, 2], [1, 2, 4], [0, 3, 4], [0, 3, 2, 4]):  # not covering, not from 0, mixing sequences, decreasing
        with pytest.raises(hg.HgError) as ei:
            hg.hg_attn_concat(w.q, w.k, w.v, w.seq_lens, w.ranges, lg, bad, w.scale)
        assert ei.value.status == -4


@pytest.mark.parametrize("index", [1, 4])
def test_full_size_sampled(index):
    """Benchmark shapes: sampled (sequence, head) pairs against the oracle, and the concat route
    against the statistics route everywhere."""
    spec = W.WORKLOADS[index]
    w = W.make_workload(spec, DEV)
    lg = hg.hg_attn_logits(w.q, w.k, w.v, w.seq_lens, w.ranges, w.scale)
    out, lse = hg.hg_attn_concat(w.q, w.k, w.v, w.seq_lens, w.ranges, lg, w.group_ptr, w.scale)
    fout, flse = hg.hg_attn_full(w.q, w.k, w.v, w.seq_lens, w.scale)
    assert (out - fout).abs().max().item() <= 2e-5 and (lse - flse).abs().max().item() <= 2e-5
    G = spec.n_q_heads // spec.n_kv_heads
    rng = np.random.RandomState(index)
    for _ in range(3):
        b, h = int(rng.randint(spec.batch)), int(rng.randint(spec.n_q_heads))
        n = int(w.seq_lens[b])
        qs = to_np(w.q[b:b + 1, h:h + 1])
        ks = to_np(w.k[b:b + 1, h // G:h // G + 1, :n])
        vs = to_np(w.v[b:b + 1, h // G:h // G + 1, :n])
        local = [(0, s, e) for (_, s, e) in w.ranges[int(w.group_ptr[b]):int(w.group_ptr[b + 1])]]
        ref = oracle.attn_concat(qs, ks, vs, [n], w.scale, local)
        rl = oracle.attn_logits(qs, ks, vs, [n], w.scale, local)
        c0 = sum(e - s for (_, s, e) in w.ranges[:int(w.group_ptr[b])])
        assert np.abs(to_np(lg[h, c0:c0 + rl.shape[1]]) - rl[0]).max() <= LOGIT_TOL
        assert np.abs(to_np(out[b, h]) - ref[0, 0]).max() <= OUT_TOL

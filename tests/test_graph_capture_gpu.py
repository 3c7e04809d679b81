"""The library enqueues kernels only (host tables travel in kernel arguments or through upload
kernels; nothing is copied, set or allocated), so a call sequence can be recorded into a HIP
graph.  The graph is replayed several times with new query values and eager work in between, and
every replay is checked against the eager result and the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_18529_amd as hg
from paper_2604_18529_amd import hg_attn as binding
from paper_2604_18529_amd import workloads as W

from parity_utils import check_out, kv_np, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("many_ranges", [False, True])
def test_partial_merge_and_full_replay_from_a_graph(many_ranges):
    hg.hg_attn_set_span_tokens(0)
    spec = W.WorkloadSpec("graph", 2, 8, 2, 128, "f16", 2000, 3000, "dirichlet", 5, seed=80)
    w = W.make_workload(spec, DEV)
    ranges, gp = w.ranges, w.group_ptr
    if many_ranges:  # more ranges and groups than fit in kernel arguments: upload kernels get recorded too
        ranges, gp = [], [0]
        for b, n in enumerate(w.seq_lens):
            for i in range(150):
                ranges.append((b, 10 * i, 10 * i + 10))
            ranges.append((b, 1500, int(n)))
            gp.append(len(ranges))
    desc, keep = hg.make_desc(w.q, w.k, w.v, w.seq_lens, w.scale)
    packed = hg.pack_ranges(ranges)
    R, Hq, d = len(ranges), spec.n_q_heads, spec.head_dim
    m = torch.empty((R, Hq), dtype=torch.float32, device=DEV)
    l = torch.empty_like(m)
    o = torch.empty((R, Hq, d), dtype=torch.float32, device=DEV)
    out = torch.empty((spec.batch, Hq, d), dtype=torch.float32, device=DEV)
    lse = torch.empty((spec.batch, Hq), dtype=torch.float32, device=DEV)
    fout, flse = torch.empty_like(out), torch.empty_like(lse)
    ws = torch.empty(max(binding.hg_attn_partial_workspace_size(desc, packed), 256), dtype=torch.uint8, device=DEV)
    fws = torch.empty(max(binding.hg_attn_full_workspace_size(desc), 256), dtype=torch.uint8, device=DEV)
    mws = torch.empty(4096, dtype=torch.uint8, device=DEV)

    def step():
        hg.hg_attn_partial(w.q, w.k, w.v, w.seq_lens, packed, w.scale, m=m, l=l, o=o, workspace=ws, desc=desc)
        hg.hg_attn_merge(m, l, o, gp, out=out, lse=lse, workspace=mws)
        hg.hg_attn_full(w.q, w.k, w.v, w.seq_lens, w.scale, out=fout, lse=flse, workspace=fws, desc=desc)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()  # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    gen = torch.Generator(device=DEV)
    gen.manual_seed(81)
    for rep in range(4):
        w.q.copy_(torch.randn(w.q.shape, generator=gen, device=DEV, dtype=torch.float32))  # new query, same buffers
        out.zero_(); fout.zero_(); m.zero_()  # eager work between the replays
        graph.replay()
        torch.cuda.synchronize()
        g_out, g_lse, g_fout = out.clone(), lse.clone(), fout.clone()
        out.zero_(); fout.zero_()
        step()  # eager, same inputs
        torch.cuda.synchronize()
        assert torch.equal(g_out, out) and torch.equal(g_lse, lse) and torch.equal(g_fout, fout), "replay %d" % rep
        ref, rlse = oracle.attn_full(to_np(w.q), *kv_np(w), w.seq_lens, w.scale)
        check_out(g_fout, flse, ref, rlse, "graph replay %d full" % rep)
        if not many_ranges:
            check_out(g_out, g_lse, ref, rlse, "graph replay %d merge" % rep)
    del keep


@pytest.mark.parametrize("mode", [1, 2])
def test_selection_flows_replay_from_a_graph(mode):
    """hg_attn_topk (filter scan: it clears its shared bounds with a fill kernel, not a memset,
    and its workgroups exchange bounds while they run; or the two-call sequence inside),
    hg_attn_gather over the kept list and hg_attn_merge2, recorded once and replayed with new
    queries: every replay equals the eager run on the same inputs, kept tokens included."""
    hg.hg_attn_set_span_tokens(1024)
    hg.hg_attn_set_topk_mode(mode)
    try:
        spec = W.WorkloadSpec("graphsel", 2, 16, 2, 128, "f16", 20000, 30000, "none", seed=82)
        w = W.make_workload(spec, DEV)
        off = [(b, 0, int(n) - 2000) for b, n in enumerate(w.seq_lens)]
        res = [(b, int(n) - 2000, int(n)) for b, n in enumerate(w.seq_lens)]
        gp = [0, 1, 2]
        desc, keep = hg.make_desc(w.q, w.k, w.v, w.seq_lens, w.scale)
        p_off, p_res = hg.pack_ranges(off), hg.pack_ranges(res)
        tws = torch.empty(binding.hg_attn_topk_workspace_size(desc, p_off, gp, 100), dtype=torch.uint8, device=DEV)
        pws = torch.empty(max(binding.hg_attn_partial_workspace_size(desc, p_res), 256), dtype=torch.uint8, device=DEV)
        out = torch.empty((2, 16, 128), dtype=torch.float32, device=DEV)
        lse = torch.empty((2, 16), dtype=torch.float32, device=DEV)

        def step():
            sel, m1, l1, o1 = hg.hg_attn_topk(w.q, w.k, w.v, w.seq_lens, p_off, gp, 100, w.scale, workspace=tws, desc=desc)
            gm, gl, go = hg.hg_attn_gather(w.q, w.k, w.v, w.seq_lens, [0, 1], sel, w.scale, desc=desc)
            m2, l2, o2 = hg.hg_attn_partial(w.q, w.k, w.v, w.seq_lens, p_res, w.scale, workspace=pws, desc=desc)
            hg.hg_attn_merge2(gm, gl, go, gp, m2, l2, o2, gp, out=out, lse=lse)
            return sel, m1, gm

        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            g_sel, g_m1, g_gm = step()
        gen = torch.Generator(device=DEV)
        gen.manual_seed(83)
        for rep in range(4):
            w.q.copy_(torch.randn(w.q.shape, generator=gen, device=DEV, dtype=torch.float32))
            out.zero_(); tws.zero_()  # eager work between the replays (the workspace may hold anything)
            graph.replay()
            torch.cuda.synchronize()
            r_sel, r_m1, r_gm, r_out, r_lse = g_sel.clone(), g_m1.clone(), g_gm.clone(), out.clone(), lse.clone()
            out.zero_()
            e_sel, e_m1, e_gm = step()
            torch.cuda.synchronize()
            assert torch.equal(r_sel, e_sel) and torch.equal(r_m1, e_m1) and torch.equal(r_gm, e_gm), "replay %d" % rep
            assert torch.equal(r_out, out) and torch.equal(r_lse, lse), "replay %d" % rep
            assert (r_m1 - r_gm).abs().max().item() <= 1e-4  # the kept maximum, computed by two different kernels
            gm, gl, go = oracle.attn_gather(to_np(w.q), *kv_np(w), w.seq_lens, w.scale, [0, 1], to_np(r_sel))
            assert np.abs(to_np(r_m1).astype(np.float64) - gm).max() <= 1e-3
        del keep
    finally:
        hg.hg_attn_set_span_tokens(0)
        hg.hg_attn_set_topk_mode(0)


def test_partial_merge_one_launch_path_replays_from_a_graph():
    """hg_attn_partial_merge on an input small enough for its one-launch path, recorded once and
    replayed with new queries: every replay equals the eager call and the oracle."""
    hg.hg_attn_set_span_tokens(0)
    w = W.make_workload(W.WORKLOADS[0], DEV)
    spec = W.WORKLOADS[0]
    desc, keep = hg.make_desc(w.q, w.k, w.v, w.seq_lens, w.scale)
    packed = hg.pack_ranges(w.ranges)
    R, Hq, d = len(w.ranges), spec.n_q_heads, spec.head_dim
    m = torch.empty((R, Hq), dtype=torch.float32, device=DEV)
    l = torch.empty_like(m)
    o = torch.empty((R, Hq, d), dtype=torch.float32, device=DEV)
    out = torch.empty((spec.batch, Hq, d), dtype=torch.float32, device=DEV)
    lse = torch.empty((spec.batch, Hq), dtype=torch.float32, device=DEV)
    ws = torch.empty(max(binding.hg_attn_partial_merge_workspace_size(desc, packed, w.group_ptr), 256), dtype=torch.uint8, device=DEV)

    def step():
        hg.hg_attn_partial_merge(w.q, w.k, w.v, w.seq_lens, packed, w.group_ptr, w.scale, m=m, l=l, o=o, out=out, lse=lse,
                                 workspace=ws, desc=desc)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    gen = torch.Generator(device=DEV)
    gen.manual_seed(84)
    for rep in range(3):
        w.q.copy_(torch.randn(w.q.shape, generator=gen, device=DEV, dtype=torch.float32))
        out.zero_(); m.zero_()
        graph.replay()
        torch.cuda.synchronize()
        g_out, g_lse, g_m = out.clone(), lse.clone(), m.clone()
        out.zero_(); m.zero_()
        step()
        torch.cuda.synchronize()
        assert torch.equal(g_out, out) and torch.equal(g_lse, lse) and torch.equal(g_m, m), "replay %d" % rep
        ref, rlse = oracle.attn_full(to_np(w.q), *kv_np(w), w.seq_lens, w.scale)
        check_out(g_out, g_lse, ref, rlse, "graph replay %d" % rep)
    del keep

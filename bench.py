#!/usr/bin/env python3
"""Benchmark of partitioned decode attention on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input that is already
resident in HBM:  hg_attn_partial over every range of every sequence (streams K and V once,
segment records, segment reduce)  ->  hg_attn_merge over each sequence's triples.

The headline workload is the largest single-GPU configuration, the OPT-30B-shaped decode layer
(batch 4, 56 heads, head_dim 128, 131072 cached tokens per sequence, fp16 K/V = 14 GiB, eight
Dirichlet partitions per sequence).  The other long-context configurations (13B-shaped ragged
batch, 1M-token grouped-query layer) get the same full measurement block under
"in_bar_workloads"; the two short configurations are reported briefly.

Prints ONE JSON line.
  value        effective KV GB/s = bytes of K and V inside the processed ranges (each row once per
               KV head) / wall time per step over exactly --steps steps, bracketed by device
               synchronisation.
  roofline     the streaming kernel alone against the 8 TB/s HBM peak: algorithmic bytes / its
               average launch duration, taken with HIP event pairs that the library records on
               the launch stream right around the kernel, during the timed steps themselves.
  timing       per-iteration event pairs over >= 100 further iterations (step and kernel in the
               same iteration): median, min, p90.
  cpu_baseline the fp64 oracle on the host cores over the same tensors, with the whole-workload
               max-abs error of the GPU result against it.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PROFILES = os.path.join(ROOT, "profiles")
HEADLINE = 3            # index into workloads.WORKLOADS: opt30b-b4-128k
IN_BAR = (2, 3, 4)      # the 32k .. 1M-token configurations the bandwidth target is stated on
PAPER_CONTEXT = (
    "paper reports only end-to-end generation speedups (1.41x-3.2x on average over six baselines; "
    "Xeon Gold 5320 + A100 80GB, Xeon Gold 6530 + H100 NVL, Xeon 6960P + RTX 5090 + CXL); "
    "no kernel-level number exists for this path"
)


def _profiled_traffic(kernel, workload, build_id):
    """HBM bytes per launch of the streaming kernel from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE, each scaled by the calibration copy) -- but only when that summary
    was taken with the very binary that is running now (it records the library's build id, a hash
    of the sources); otherwise None: a counter reading of other code is not this run's traffic."""
    path = os.path.join(PROFILES, "%s__%s.md" % (kernel, workload))
    traffic, prof_id = None, None
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = float(line.split(":", 1)[1])
            if line.startswith("library_build_id:"):
                prof_id = line.split(":", 1)[1].strip()
    except OSError:
        return None, None
    if traffic is None or prof_id != build_id:
        return None, "%s (taken with build %s, running %s: ignored)" % (os.path.relpath(path, ROOT), prof_id, build_id)
    return traffic, os.path.relpath(path, ROOT)


def _stats(xs, scale=1.0):
    s = sorted(xs)
    n = len(s)
    if n == 0:
        return None
    return {"median": s[n // 2] * scale, "min": s[0] * scale, "p90": s[min(n - 1, (9 * n) // 10)] * scale,
            "mean": sum(s) / n * scale, "n": n}


def _time_loop(step, steps, warmup, torch):
    """Exactly `steps` steps between two device synchronisations; milliseconds per step by events."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return e0.elapsed_time(e1) / steps, wall_ms / steps


def _settle(step, settle_ms, torch):
    """Untimed: keep the device under this step's load for settle_ms before anything is timed.
    Measured on MI355X, the first 0.2 s of sustained streaming after a pause run about 5 % slower
    than what follows (the kernel's duration along a 200-step loop that started cold: 2206, 2180,
    2154, 2172, 2097, 2098, 2097 ... us per tenth), so a timed region that starts cold mixes two
    regimes.  The timed steps themselves are unchanged."""
    if settle_ms <= 0:
        return
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < settle_ms:
        for _ in range(8):
            step()
        torch.cuda.synchronize()


def _time_each(step, iters, warmup, torch, hg):
    """`iters` iterations, each with its own event pair around the step and (recorded by the
    library on the same stream) around the streaming kernel inside it.  Returns two lists of
    milliseconds: per step, per kernel launch."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    hg.hg_attn_profile_start(iters, 1)
    for a, b in ev:
        a.record()
        step()
        b.record()
    torch.cuda.synchronize()
    kernel_ms = hg.hg_attn_profile_times(iters)
    hg.hg_attn_profile_stop()
    return [a.elapsed_time(b) for a, b in ev], kernel_ms


def _kernel_name(spec):
    if spec.dtype != "f32" and spec.n_q_heads // spec.n_kv_heads >= 2:  # the library's own dispatch rule
        return "hg_partial_gqa_kernel" if spec.head_dim == 128 else "hg_partial_gqa64_kernel"
    return "hg_partial_kernel"


def _cpu_baseline(w, spec, step, out, torch):
    """The oracle as it stands on the host cores, over the whole workload (partial per range +
    merge: the same decomposition the GPU step runs), and the GPU result's error against it."""
    import numpy as np

    import oracle

    def host(t):
        t = t.cpu()
        return t.view(torch.int16).numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.numpy()

    qn, kn, vn = host(w.q), host(w.k), host(w.v)
    threads = oracle.max_threads()
    step()
    torch.cuda.synchronize()
    gpu_out = out.cpu().numpy()
    t0 = time.perf_counter()
    mo, lo, oo = oracle.attn_partial(qn, kn, vn, w.seq_lens, w.scale, w.ranges)
    ref, _ = oracle.attn_merge(mo, lo, oo, w.group_ptr)
    secs = time.perf_counter() - t0
    err = float(np.abs(gpu_out - ref).max())
    del qn, kn, vn
    return {
        "value": w.kv_bytes / secs / 1e9,
        "unit": "GB/s",
        "cores": threads,
        "kind": "oracle",
        "sample": "whole workload %s, every (sequence, head): fp64 partial statistics per range + merge, once; "
                  "OpenMP over (range, head); %.1f s = %.0f core-seconds" % (spec.name, secs, secs * threads),
        "seconds": secs,
        "gpu_max_abs_err_vs_oracle": err,
        "error_covers": "all %d x %d (sequence, head) outputs" % (spec.batch, spec.n_q_heads),
    }


def _routes(w, spec, steps, warmup, torch, hg, W, binding, desc, packed, out, lse, ws):
    """Timings of the widened rows on the same tensors: the paper-literal concat route, the
    Post-QK^T and Pre-QK^T flows, a paged cache, and proxy-query partitions with their error."""
    dev = w.q.device
    Hq, d = spec.n_q_heads, spec.head_dim
    n = max(steps, 1)
    wu = max(warmup, 1)
    ltok = sum(e - b for (_, b, e) in w.ranges)
    logits = torch.empty((Hq, ltok), dtype=torch.float32, device=dev)
    cws = torch.empty(max(binding.hg_attn_concat_workspace_size(desc, packed, spec.batch), 256), dtype=torch.uint8, device=dev)

    def logits_step():
        hg.hg_attn_logits(w.q, w.k, w.v, w.seq_lens, packed, w.scale, logits=logits, desc=desc)

    def concat_step():
        hg.hg_attn_concat(w.q, w.k, w.v, w.seq_lens, packed, logits, w.group_ptr, w.scale, out=out, lse=lse,
                          workspace=cws, desc=desc)

    logits_ms, _ = _time_loop(logits_step, n, wu, torch)
    concat_ms, _ = _time_loop(concat_step, n, wu, torch)

    # Post-QK^T flow: logits of the offloaded 80 % of every cache, top-128 per (sequence, head),
    # triple of the kept tokens; the resident 20 % streamed as usual; one merge
    old = [(b, 0, int(0.8 * n_b)) for b, n_b in enumerate(w.seq_lens)]
    new = [(b, int(0.8 * n_b), int(n_b)) for b, n_b in enumerate(w.seq_lens)]
    p_old, p_new = hg.pack_ranges(old), hg.pack_ranges(new)
    gp_old = list(range(spec.batch + 1))
    one_each = list(range(spec.batch + 1))
    nws = torch.empty(max(binding.hg_attn_partial_workspace_size(desc, p_new), 256), dtype=torch.uint8, device=dev)
    ows = torch.empty(max(binding.hg_attn_partial_workspace_size(desc, p_old), 256), dtype=torch.uint8, device=dev)
    top_k = 128
    tws = torch.empty(max(binding.hg_attn_topk_workspace_size(desc, p_old, gp_old, top_k), 256), dtype=torch.uint8, device=dev)

    def postqk_topk():
        return hg.hg_attn_topk(w.q, w.k, w.v, w.seq_lens, p_old, gp_old, top_k, w.scale, want_sel=False, workspace=tws, desc=desc)

    def postqk_step():
        _, m1, l1, o1 = postqk_topk()
        m2, l2, o2 = hg.hg_attn_partial(w.q, w.k, w.v, w.seq_lens, p_new, w.scale, workspace=nws, desc=desc)
        hg.hg_attn_merge2(m1, l1, o1, one_each, m2, l2, o2, one_each, out=out, lse=lse)

    pq_topk_ms, _ = _time_loop(postqk_topk, n, wu, torch)
    pq_step_ms, _ = _time_loop(postqk_step, n, wu, torch)

    # Pre-QK^T flow: 128 listed tokens per (sequence, head) of the offloaded part (a seeded stand-in
    # for the selector), evaluated with hg_attn_gather; resident 20 % and merge as above
    lists = torch.from_numpy(W.listed_tokens([e for (_, _, e) in old], Hq, top_k, seed=11)).to(dev)
    seq_of_group = list(range(spec.batch))
    gm = torch.empty((spec.batch, Hq), dtype=torch.float32, device=dev)
    gl = torch.empty((spec.batch, Hq), dtype=torch.float32, device=dev)
    go = torch.empty((spec.batch, Hq, d), dtype=torch.float32, device=dev)

    def preqk_step():
        m1, l1, o1 = hg.hg_attn_gather(w.q, w.k, w.v, w.seq_lens, seq_of_group, lists, w.scale, m=gm, l=gl, o=go,
                                       workspace=ws, desc=desc)
        m2, l2, o2 = hg.hg_attn_partial(w.q, w.k, w.v, w.seq_lens, p_new, w.scale, workspace=nws, desc=desc)
        hg.hg_attn_merge2(m1, l1, o1, one_each, m2, l2, o2, one_each, out=out, lse=lse)

    pre_step_ms, _ = _time_loop(preqk_step, n, wu, torch)

    # Proxy-query partitions: the offloaded 80 % is scanned with an approximate query (the true one
    # rotated to a given cosine similarity: a stand-in for the previous layer's input pushed through
    # this layer's weights), the resident 20 % with the true query; exact merge of the two.  The
    # error is against exact attention (hg_attn_full on the same tensors).
    exact = torch.empty_like(out)
    fws = torch.empty(max(binding.hg_attn_full_workspace_size(desc), 256), dtype=torch.uint8, device=dev)
    hg.hg_attn_full(w.q, w.k, w.v, w.seq_lens, w.scale, out=exact, want_lse=False, workspace=fws, desc=desc)
    proxy = {}
    for cosine in (0.98, 0.9):
        qp = W.proxy_query(w.q, cosine, seed=7)
        pdesc, pkeep = hg.make_desc(qp, w.k, w.v, w.seq_lens, w.scale)
        pout = torch.empty_like(out)

        def proxy_step():
            m1, l1, o1 = hg.hg_attn_partial(qp, w.k, w.v, w.seq_lens, p_old, w.scale, workspace=ows, desc=pdesc)
            m2, l2, o2 = hg.hg_attn_partial(w.q, w.k, w.v, w.seq_lens, p_new, w.scale, workspace=nws, desc=desc)
            hg.hg_attn_merge2(m1, l1, o1, one_each, m2, l2, o2, one_each, out=pout, want_lse=False)

        pms, _ = _time_loop(proxy_step, n, wu, torch)
        proxy["cosine_%.2f" % cosine] = {"us": pms * 1e3, "max_abs_err_vs_exact": float((pout - exact).abs().max()),
                                         "mean_abs_err_vs_exact": float((pout - exact).abs().mean())}
        del pdesc, pkeep

    # the same cache as a paged pool (256-token blocks in shuffled physical order), same step
    kp, vp, table = W.make_paged(w, 256, seed=1)
    gdesc, gkeep = hg.make_desc(w.q, kp, vp, w.seq_lens, w.scale, table)
    pws = torch.empty(max(binding.hg_attn_partial_workspace_size(gdesc, packed), 256), dtype=torch.uint8, device=dev)
    R = len(w.ranges)
    m = torch.empty((R, Hq), dtype=torch.float32, device=dev)
    l = torch.empty((R, Hq), dtype=torch.float32, device=dev)
    o = torch.empty((R, Hq, d), dtype=torch.float32, device=dev)

    def paged_step():
        hg.hg_attn_partial(w.q, kp, vp, w.seq_lens, packed, w.scale, m=m, l=l, o=o, workspace=pws, desc=gdesc)
        hg.hg_attn_merge(m, l, o, w.group_ptr, out=out, lse=lse)

    paged_ms, _ = _time_loop(paged_step, n, wu, torch)
    del kp, vp, table, gdesc, gkeep
    k_bytes = w.kv_bytes // 2
    return {
        "steps_each": n,
        "concat_route": {"logits_us": logits_ms * 1e3, "concat_us": concat_ms * 1e3, "us": (logits_ms + concat_ms) * 1e3,
                         "logits_bytes": Hq * ltok * 4,
                         "logits_gbps_on_k_bytes": k_bytes / (logits_ms * 1e-3) / 1e9,
                         "logits_gbps_on_bytes_moved": (k_bytes + Hq * ltok * 4) / (logits_ms * 1e-3) / 1e9,
                         "concat_gbps_on_bytes_moved": (k_bytes + Hq * ltok * 4) / (concat_ms * 1e-3) / 1e9},  # V + the logits
        "post_qk_route": {"offloaded_fraction": 0.8, "top_k": top_k, "topk_us": pq_topk_ms * 1e3, "us": pq_step_ms * 1e3},
        "pre_qk_route": {"offloaded_fraction": 0.8, "listed_tokens": top_k, "us": pre_step_ms * 1e3},
        "proxy_query": dict(proxy, offloaded_fraction=0.8),
        "paged_cache_block_256": {"us": paged_ms * 1e3, "gbps": w.kv_bytes / (paged_ms * 1e-3) / 1e9},
    }


def run_workload(index, torch, hg, W, *, steps=0, warmup=0, iters=100, cpu_baseline=True, routes=False, route_steps=20,
                 settle_ms=0):
    """Full measurement block of one workload.  steps > 0: also the bracketed loop of exactly
    `steps` steps (the headline), with the kernel's event pairs recorded during those steps."""
    from paper_2604_18529_amd import hg_attn as binding

    spec = W.ALL_WORKLOADS[index]
    w = W.make_workload(spec, "cuda:0")
    desc, keep = hg.make_desc(w.q, w.k, w.v, w.seq_lens, w.scale)
    packed = hg.pack_ranges(w.ranges)
    R = len(w.ranges)
    dev = w.q.device
    Hq, d = spec.n_q_heads, spec.head_dim
    m = torch.empty((R, Hq), dtype=torch.float32, device=dev)
    l = torch.empty((R, Hq), dtype=torch.float32, device=dev)
    o = torch.empty((R, Hq, d), dtype=torch.float32, device=dev)
    out = torch.empty((spec.batch, Hq, d), dtype=torch.float32, device=dev)
    lse = torch.empty((spec.batch, Hq), dtype=torch.float32, device=dev)
    ws = torch.empty(max(binding.hg_attn_partial_workspace_size(desc, packed), 256), dtype=torch.uint8, device=dev)
    span_tokens, n_workgroups = hg.hg_attn_plan(w.q, w.k, w.v, w.seq_lens, packed, w.scale)
    kv_bytes = w.kv_bytes

    def step():
        hg.hg_attn_partial(w.q, w.k, w.v, w.seq_lens, packed, w.scale, m=m, l=l, o=o, workspace=ws, desc=desc)
        hg.hg_attn_merge(m, l, o, w.group_ptr, out=out, lse=lse)

    res = {
        "workload": spec.name, "batch": spec.batch, "n_q_heads": Hq, "n_kv_heads": spec.n_kv_heads, "head_dim": d,
        "kv_dtype": spec.dtype, "tokens_total": int(w.seq_lens.sum()), "partitions": R, "span_tokens": span_tokens,
        "workgroups": n_workgroups, "kv_bytes": kv_bytes,
    }
    loop_kernel_ms = None
    _settle(step, settle_ms, torch)
    if steps > 0:
        # the headline loop: kernel event pairs are recorded by the library during these very steps
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        hg.hg_attn_profile_start(steps, 1)
        ms, wall_ms = _time_loop(step, steps, 0, torch)
        loop_kernel_ms = hg.hg_attn_profile_times(steps)
        hg.hg_attn_profile_stop()
        res.update({"loop_ms_per_step": ms, "loop_host_wall_ms_per_step": wall_ms})
        # the kernel's duration along the timed loop (every tenth of it), to show drift
        tenth = max(len(loop_kernel_ms) // 10, 1)
        res["loop_kernel_us_by_tenth"] = [round(sum(loop_kernel_ms[i:i + tenth]) / len(loop_kernel_ms[i:i + tenth]) * 1e3, 1)
                                          for i in range(0, len(loop_kernel_ms), tenth)][:10]

    step_ms, kernel_ms = _time_each(step, iters, max(warmup, 5), torch, hg)
    st, kt = _stats(step_ms, 1e3), _stats(kernel_ms, 1e3)
    res["step_us"] = st
    res["stream_kernel_us"] = kt
    us = ms * 1e3 if steps > 0 else st["median"]
    res["us_per_layer"] = us
    res["gbps"] = kv_bytes / (us * 1e-6) / 1e9
    res["frac_hbm_peak"] = res["gbps"] / HBM_PEAK_GBS
    res["kernel_le_step_every_iteration"] = all(k <= s for k, s in zip(kernel_ms, step_ms))

    # roofline of the streaming kernel: average launch duration over the timed region (the
    # headline loop when there is one, else the per-iteration pass)
    avg_kernel_ms = sum(loop_kernel_ms) / len(loop_kernel_ms) if loop_kernel_ms else sum(kernel_ms) / len(kernel_ms)
    kname = _kernel_name(spec)
    traffic, traffic_src = _profiled_traffic(kname, spec.name, hg.hg_attn_build_id())
    res["roofline"] = {
        "bound": "hbm", "kernel": kname, "achieved": kv_bytes / (avg_kernel_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
        "unit": "GB/s", "frac": kv_bytes / (avg_kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": traffic,
        "traffic_source": traffic_src, "kernel_us_avg": avg_kernel_ms * 1e3, "kernel_us_median": kt["median"],
        "kernel_us_min": kt["min"], "frac_at_median": kv_bytes / (kt["median"] * 1e-6) / 1e9 / HBM_PEAK_GBS,
        "launches_timed": len(loop_kernel_ms) if loop_kernel_ms else len(kernel_ms),
        "algorithmic_bytes_per_launch": kv_bytes,
        "bytes_per_unit": "512 B per cached token per KV head (K row + V row, head_dim 128 fp16) x %d tokens x %d KV heads"
                          % (int(w.seq_lens.sum()), spec.n_kv_heads) if d * w.k.element_size() == 256 else
                          "%d B per cached token per KV head x %d tokens x %d KV heads"
                          % (2 * d * w.k.element_size(), int(w.seq_lens.sum()), spec.n_kv_heads),
    }

    # the unsplit path, for reference
    fws = torch.empty(max(binding.hg_attn_full_workspace_size(desc), 256), dtype=torch.uint8, device=dev)

    def full_step():
        hg.hg_attn_full(w.q, w.k, w.v, w.seq_lens, w.scale, out=out, lse=lse, workspace=fws, desc=desc)

    full_ms, _ = _time_loop(full_step, max(iters // 4, 5), 3, torch)
    res["full_path_us"] = full_ms * 1e3

    if steps > 0:
        # the same step recorded once into a HIP graph and replayed
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            step()
        graph_ms, _ = _time_loop(graph.replay, max(iters // 2, 10), 3, torch)
        res["graph_replay_us"] = graph_ms * 1e3
        del graph

    if routes:
        res["routes"] = _routes(w, spec, route_steps, 3, torch, hg, W, binding, desc, packed, out, lse, ws)
    if cpu_baseline:
        res["cpu_baseline"] = _cpu_baseline(w, spec, step, out, torch)
    del keep
    return res


def run_tiny(torch, hg, W, iters=200, sets=64):
    """The tiny configuration is launch-bound (1 MiB of K and V): microseconds only, rotating over
    `sets` distinct copies of the tensors so that no iteration finds its input in a cache."""
    from paper_2604_18529_amd import hg_attn as binding

    spec = W.WORKLOADS[0]
    w = W.make_workload(spec, "cuda:0")
    packed = hg.pack_ranges(w.ranges)
    copies = []
    for _ in range(sets):
        q, k, v = w.q.clone(), w.k.clone(), w.v.clone()
        desc, keep = hg.make_desc(q, k, v, w.seq_lens, w.scale)
        copies.append((q, k, v, desc, keep))
    R, Hq, d = len(w.ranges), spec.n_q_heads, spec.head_dim
    dev = w.q.device
    m = torch.empty((R, Hq), dtype=torch.float32, device=dev)
    l = torch.empty((R, Hq), dtype=torch.float32, device=dev)
    o = torch.empty((R, Hq, d), dtype=torch.float32, device=dev)
    out = torch.empty((spec.batch, Hq, d), dtype=torch.float32, device=dev)
    ws = torch.empty(max(binding.hg_attn_partial_workspace_size(copies[0][3], packed), 256), dtype=torch.uint8, device=dev)
    fws = torch.empty(max(binding.hg_attn_full_workspace_size(copies[0][3]), 256), dtype=torch.uint8, device=dev)
    turn = [0]

    def step():
        q, k, v, desc, _ = copies[turn[0] % sets]
        turn[0] += 1
        hg.hg_attn_partial(q, k, v, w.seq_lens, packed, w.scale, m=m, l=l, o=o, workspace=ws, desc=desc)
        hg.hg_attn_merge(m, l, o, w.group_ptr, out=out, want_lse=False)

    def full_step():
        q, k, v, desc, _ = copies[turn[0] % sets]
        turn[0] += 1
        hg.hg_attn_full(q, k, v, w.seq_lens, w.scale, out=out, want_lse=False, workspace=fws, desc=desc)

    pws = torch.empty(max(binding.hg_attn_partial_merge_workspace_size(copies[0][3], packed, w.group_ptr), 256), dtype=torch.uint8,
                      device=dev)

    def one_call_step():  # the same outputs through hg_attn_partial_merge: one launch at this size
        q, k, v, desc, _ = copies[turn[0] % sets]
        turn[0] += 1
        hg.hg_attn_partial_merge(q, k, v, w.seq_lens, packed, w.group_ptr, w.scale, m=m, l=l, o=o, out=out, want_lse=False,
                                 workspace=pws, desc=desc)

    step_ms, kernel_ms = _time_each(step, iters, 10, torch, hg)
    full_ms, _ = _time_each(full_step, iters, 10, torch, hg)
    one_ms, _ = _time_each(one_call_step, iters, 10, torch, hg)
    return {"workload": spec.name, "kv_bytes": w.kv_bytes, "buffer_sets": sets, "step_us": _stats(step_ms, 1e3),
            "stream_kernel_us": _stats(kernel_ms, 1e3), "full_path_us": _stats(full_ms, 1e3),
            "partial_merge_one_call_us": _stats(one_ms, 1e3),
            "note": "launch-bound: three launches per step (one for the unsplit path and for hg_attn_partial_merge); microseconds only"}


def run_memory_probe(torch, hg, read_bytes=7516192768, reps=5):
    """What this memory system gives a one-pass read stream with the streaming kernels' access
    pattern, alone and next to writes (hg_attn_calibration_stream): the practical ceiling the
    kernels are tuned against, and the cost of writes that trickle out next to the stream against
    writes that go out in rare bursts.  read_bytes defaults to the K bytes of opt30b-b4-128k."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    src = torch.zeros(read_bytes + cus * 32768 + 65536, dtype=torch.uint8, device="cuda:0")
    dst = torch.zeros(read_bytes // 8 + (1 << 20), dtype=torch.uint8, device="cuda:0")
    iters = read_bytes // 16 // cus // 2048  # workgroup iterations of 32 KiB
    rows = []

    def timed(wvec, burst, nt):
        def call():
            hg.hg_attn_calibration_stream(src, read_bytes, dst, wvec, burst, nt)
        ms, _ = _time_loop(call, reps, 2, torch)
        written = (iters // burst) * burst * wvec * 16 * cus if wvec else 0
        rows.append({"write_share": "none" if not wvec else "1/%d of the bytes" % (2048 // wvec), "burst_iterations": burst if wvec else None,
                     "streaming_stores": bool(nt) if wvec else None, "written_bytes": written, "us": ms * 1e3,
                     "read_gbps": iters * cus * 32768 / (ms * 1e-3) / 1e9})

    timed(0, 1, 0)
    for wvec in (32, 256):
        for burst in (1, 16, 64, 128, 224, 448):
            for nt in (0, 1):
                timed(wvec, burst, nt)
    timed(0, 1, 0)
    return {"read_bytes": iters * cus * 32768, "workgroups": cus, "iterations_per_workgroup": iters, "rows": rows}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=HEADLINE,
                    help="headline workload: index into workloads.ALL_WORKLOADS (default 3, the largest single-GPU configuration)")
    ap.add_argument("--others", type=str, default="2,4,1,0",
                    help="comma list of further workloads: the in-bar ones (2, 3, 4) get the full block, 1 a short one, 0 the tiny one ('' for none)")
    ap.add_argument("--iters", type=int, default=100, help="iterations of the per-iteration timing pass (>= 100 by default)")
    ap.add_argument("--settle-ms", type=float, default=400.0,
                    help="untimed milliseconds of the step's own load before the warm-up steps of every workload (0: none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--routes", choices=("none", "headline", "all"), default="headline",
                    help="time the widened rows (concat, Post-QK^T, Pre-QK^T, proxy query, paged cache) on the headline workload, on every in-bar workload, or not at all")
    ap.add_argument("--span-tokens", type=int, default=0, help="force the span length (tuning)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run the library's plain 1 GiB device copy three times (known traffic: the "
                         "yardstick profiler byte counters are scaled by)")
    ap.add_argument("--memory-probe", action="store_true",
                    help="only run the plain read stream next to writes (hg_attn_calibration_stream) and print its table")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures one GPU only (across GPUs the path shards by (sequence, KV head), "
                 "or by token range with one exchange of the (m, l, O) triples); run with --gpus 1")

    import torch

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    import paper_2604_18529_amd as hg
    from paper_2604_18529_amd import workloads as W

    hg.load_library()
    hg.hg_attn_set_span_tokens(args.span_tokens)

    if args.memory_probe:
        print(json.dumps({"memory_probe": run_memory_probe(torch, hg), "library_build_id": hg.hg_attn_build_id()}))
        return

    if args.calibration_copy:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            hg.hg_attn_calibration_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    cpu = not args.no_cpu_baseline
    head = run_workload(args.workload, torch, hg, W, steps=args.steps, warmup=args.warmup, iters=args.iters, cpu_baseline=cpu,
                        routes=args.routes != "none", settle_ms=args.settle_ms)
    in_bar, short = [], []
    for tok in [t for t in args.others.split(",") if t.strip()]:
        i = int(tok)
        if i == args.workload:
            continue
        # (No torch.cuda.empty_cache() between workloads: memory handed back to the driver and
        # allocated again is placed worse.  Measured in one run, the streaming kernel on the ragged
        # and the 1M-token workload: 85.0 % / 82.2 % of the HBM peak on tensors allocated after the
        # headline's route buffers had been freed to the driver, 90.0 % / 88.1 % when the caching
        # allocator serves them from the blocks it kept.  288 GB hold every workload's tensors.)
        if i == 0:
            short.append(run_tiny(torch, hg, W))
        elif i in IN_BAR:
            in_bar.append(run_workload(i, torch, hg, W, iters=args.iters, cpu_baseline=cpu, routes=args.routes == "all",
                                       settle_ms=args.settle_ms))
        else:
            # (a loop of 200 steps as well: between 150-us kernels the event pairs of the
            # per-iteration pass cost a visible share of the step)
            r = run_workload(i, torch, hg, W, steps=200, warmup=20, iters=args.iters, cpu_baseline=False, routes=False,
                             settle_ms=args.settle_ms)
            short.append({k: r[k] for k in ("workload", "kv_bytes", "us_per_layer", "gbps", "frac_hbm_peak", "step_us",
                                            "stream_kernel_us", "full_path_us", "graph_replay_us")})

    # The headline's bracketed loop once more at the end of the process, for diagnosis only
    # (`value` is the first one): on some machines, for hours at a time, whichever workload came
    # first in a process ran 5-6 % below what the same workload reached later in the same process.
    again = None
    if in_bar or short:
        r = run_workload(args.workload, torch, hg, W, steps=args.steps, warmup=args.warmup, iters=20, cpu_baseline=False,
                         routes=False, settle_ms=args.settle_ms)
        again = {"us_per_layer": r["us_per_layer"], "gbps": r["gbps"], "frac_hbm_peak": r["frac_hbm_peak"],
                 "note": "the headline's timed loop repeated after the other workloads, on tensors re-created from the "
                         "allocator's cache (on a healthy machine 1-2 % below the first measurement); not used for `value`"}

    line = {
        "metric": "decode attention effective KV GB/s (% of HBM peak) and us/layer at 1 GPU",
        "value": head["gbps"],
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle_ms": args.settle_ms,  # untimed load before the warm-up steps (see _settle)
        "ms_per_step": head["us_per_layer"] / 1e3,
        "us_per_layer": head["us_per_layer"],
        "frac_hbm_peak": head["frac_hbm_peak"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",      # the arithmetic type: products, sums, exponentials, triples and outputs
        "kv_dtype": head["kv_dtype"],  # the storage type of q, K and V
        "data": "synthetic",
        "config": {k: head[k] for k in ("workload", "batch", "n_q_heads", "n_kv_heads", "head_dim", "kv_dtype",
                                        "tokens_total", "partitions", "span_tokens", "workgroups", "kv_bytes")},
        "roofline": head["roofline"],
        "cpu_baseline": head.get("cpu_baseline"),
        "timing": {k: head.get(k) for k in ("step_us", "stream_kernel_us", "kernel_le_step_every_iteration", "full_path_us",
                                            "graph_replay_us", "loop_host_wall_ms_per_step", "loop_kernel_us_by_tenth")},
        "headline_again_at_the_end": again,
        "in_bar_workloads": in_bar,
        "short_workloads": short,
        "routes": head.get("routes"),
        "library_build_id": hg.hg_attn_build_id(),
        "paper_context": PAPER_CONTEXT,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()

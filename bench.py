#!/usr/bin/env python3
"""Benchmark of partitioned decode attention on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input that is already
resident in HBM:  hg_attn_partial over every range of every sequence (streams K and V once,
segment records, segment reduce)  ->  hg_attn_merge over each sequence's triples.  The headline
workload is the OPT-6.7B-shaped decode layer (batch 8, 32 heads, head_dim 128, 8192 cached
tokens per sequence, fp16 K/V, two partitions per sequence); the longer workloads are timed the
same way and reported under "other_workloads".

Prints ONE JSON line.  `value` = effective KV GB/s = bytes of K and V inside the processed
ranges (each row once per KV head) / wall time per step.  `roofline` prices the streaming
kernel alone against the 8 TB/s HBM peak, timed with HIP events recorded around its launches.
`cpu_baseline` is the fp64 oracle on the host cores over the same tensors.
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


def _profiled_traffic(kernel, workload):
    """HBM bytes per launch of the streaming kernel as measured by the committed rocprofv3 --pmc
    runs (FETCH_SIZE + WRITE_SIZE, each scaled by the calibration copy); None if no summary."""
    path = os.path.join(PROFILES, "%s__%s.md" % (kernel, workload))
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1]), os.path.relpath(path, ROOT)
    except OSError:
        pass
    return None, None
PAPER_CONTEXT = (
    "paper reports only end-to-end generation speedups (1.41x-3.2x on average over six baselines; "
    "Xeon Gold 5320 + A100 80GB, Xeon Gold 6530 + H100 NVL, Xeon 6960P + RTX 5090 + CXL); "
    "no kernel-level number exists for this path"
)


def _time_steps(step, steps, warmup, torch):
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


def run_workload(index, steps, warmup, with_cpu_baseline, torch, hg, W, routes=True, loops=1):
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
    from paper_2604_18529_amd import hg_attn as binding

    ws = torch.empty(max(binding.hg_attn_partial_workspace_size(desc, packed), 256), dtype=torch.uint8, device=dev)
    span_tokens, n_workgroups = hg.hg_attn_plan(w.q, w.k, w.v, w.seq_lens, packed, w.scale)

    def step():
        hg.hg_attn_partial(w.q, w.k, w.v, w.seq_lens, packed, w.scale, m=m, l=l, o=o, workspace=ws, desc=desc)
        hg.hg_attn_merge(m, l, o, w.group_ptr, out=out, lse=lse)

    # the headline workload times exactly `steps` steps once; the other workloads take the better
    # of `loops` such loops
    ms, wall_ms = min(_time_steps(step, steps, warmup, torch) for _ in range(loops))

    # the same step recorded once into a HIP graph and replayed: what a serving loop would do
    # to take the host's launch cost out of short layers
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        step()
    graph_ms, _ = _time_steps(graph.replay, steps, warmup, torch)

    # second pass of the same K steps with event pairs around the streaming kernel alone
    # (8 back-to-back launches per pair, so the cost of the event records is amortised)
    hg.hg_attn_profile_start(steps, 8)
    for _ in range(steps):
        step()
    kernel_ms_total, launches = hg.hg_attn_profile_stop()
    kernel_ms = kernel_ms_total / max(launches, 1)

    # the unsplit path, for reference
    fws = torch.empty(max(binding.hg_attn_full_workspace_size(desc), 256), dtype=torch.uint8, device=dev)

    def full_step():
        hg.hg_attn_full(w.q, w.k, w.v, w.seq_lens, w.scale, out=out, lse=lse, workspace=fws, desc=desc)

    full_ms, _ = _time_steps(full_step, max(steps // 2, 1), max(warmup // 2, 1), torch)

    kv_bytes = w.kv_bytes
    route_results = {}
    if routes:
        # the paper-literal route: export raw logits per range, then concatenate, one softmax, P.V
        ltok = sum(e - b for (_, b, e) in w.ranges)
        logits = torch.empty((Hq, ltok), dtype=torch.float32, device=dev)
        cws = torch.empty(max(binding.hg_attn_concat_workspace_size(desc, packed, spec.batch), 256), dtype=torch.uint8, device=dev)

        def logits_step():
            hg.hg_attn_logits(w.q, w.k, w.v, w.seq_lens, packed, w.scale, logits=logits, desc=desc)

        def concat_step():
            hg.hg_attn_concat(w.q, w.k, w.v, w.seq_lens, packed, logits, w.group_ptr, w.scale, out=out, lse=lse,
                              workspace=cws, desc=desc)

        logits_ms, _ = _time_steps(logits_step, max(steps // 2, 1), max(warmup // 2, 1), torch)
        concat_ms, _ = _time_steps(concat_step, max(steps // 2, 1), max(warmup // 2, 1), torch)

        # Post-QK^T flow (the paper's default selection mode): logits of the offloaded 80 % of every
        # cache, top-128 per (sequence, head), triple of the kept tokens; the resident 20 % streamed
        # as usual; one merge
        old = [(b, 0, int(0.8 * n)) for b, n in enumerate(w.seq_lens)]
        new = [(b, int(0.8 * n), int(n)) for b, n in enumerate(w.seq_lens)]
        p_old, p_new = hg.pack_ranges(old), hg.pack_ranges(new)
        lg_old = torch.empty((Hq, sum(e - b for (_, b, e) in old)), dtype=torch.float32, device=dev)
        gp_old = list(range(spec.batch + 1))
        one_each = list(range(spec.batch + 1))  # per sequence: one triple from the selection, one from the resident part
        nws = torch.empty(max(binding.hg_attn_partial_workspace_size(desc, p_new), 256), dtype=torch.uint8, device=dev)
        top_k = 128

        def postqk_logits():
            hg.hg_attn_logits(w.q, w.k, w.v, w.seq_lens, p_old, w.scale, logits=lg_old, desc=desc)

        def postqk_select():
            return hg.hg_attn_select(w.q, w.k, w.v, w.seq_lens, p_old, lg_old, gp_old, top_k, w.scale, want_sel=False, desc=desc)

        def postqk_rest():
            _, m1, l1, o1 = postqk_select()
            m2, l2, o2 = hg.hg_attn_partial(w.q, w.k, w.v, w.seq_lens, p_new, w.scale, workspace=nws, desc=desc)
            hg.hg_attn_merge2(m1, l1, o1, one_each, m2, l2, o2, one_each, out=out, lse=lse)

        tws = torch.empty(max(binding.hg_attn_topk_workspace_size(desc, p_old, gp_old, top_k), 256), dtype=torch.uint8, device=dev)

        def postqk_topk():
            return hg.hg_attn_topk(w.q, w.k, w.v, w.seq_lens, p_old, gp_old, top_k, w.scale, want_sel=False, workspace=tws, desc=desc)

        def postqk_fused_step():
            _, m1, l1, o1 = postqk_topk()
            m2, l2, o2 = hg.hg_attn_partial(w.q, w.k, w.v, w.seq_lens, p_new, w.scale, workspace=nws, desc=desc)
            hg.hg_attn_merge2(m1, l1, o1, one_each, m2, l2, o2, one_each, out=out, lse=lse)

        pq_topk_ms, _ = _time_steps(postqk_topk, max(steps // 4, 1), max(warmup // 4, 1), torch)
        pq_fused_ms, _ = _time_steps(postqk_fused_step, max(steps // 4, 1), max(warmup // 4, 1), torch)
        pq_logits_ms, _ = _time_steps(postqk_logits, max(steps // 4, 1), max(warmup // 4, 1), torch)
        pq_select_ms, _ = _time_steps(postqk_select, max(steps // 4, 1), max(warmup // 4, 1), torch)
        pq_rest_ms, _ = _time_steps(postqk_rest, max(steps // 4, 1), max(warmup // 4, 1), torch)

        # Pre-QK^T flow: the tokens of the offloaded 80 % are named up front (a seeded stand-in for
        # the selector: 128 distinct positions per (sequence, head)); the executor evaluates exactly
        # those with hg_attn_gather; resident 20 % and merge as above
        lists = torch.from_numpy(W.listed_tokens([e for (_, _, e) in old], Hq, top_k, seed=11)).to(dev)
        seq_of_group = list(range(spec.batch))

        gm = torch.empty((spec.batch, Hq), dtype=torch.float32, device=dev)
        gl = torch.empty((spec.batch, Hq), dtype=torch.float32, device=dev)
        go = torch.empty((spec.batch, Hq, d), dtype=torch.float32, device=dev)

        def preqk_gather():
            return hg.hg_attn_gather(w.q, w.k, w.v, w.seq_lens, seq_of_group, lists, w.scale, m=gm, l=gl, o=go,
                                     workspace=ws, desc=desc)

        def preqk_step():
            m1, l1, o1 = preqk_gather()
            m2, l2, o2 = hg.hg_attn_partial(w.q, w.k, w.v, w.seq_lens, p_new, w.scale, workspace=nws, desc=desc)
            hg.hg_attn_merge2(m1, l1, o1, one_each, m2, l2, o2, one_each, out=out, lse=lse)

        pre_gather_ms, _ = _time_steps(preqk_gather, max(steps // 4, 1), max(warmup // 4, 1), torch)
        pre_step_ms, _ = _time_steps(preqk_step, max(steps // 4, 1), max(warmup // 4, 1), torch)

        # the same cache as a paged pool (16-token blocks in shuffled physical order), same step
        paged = {}
        for bt in (16, 256):
            kp, vp, table = W.make_paged(w, bt, seed=1)
            pdesc, pkeep = hg.make_desc(w.q, kp, vp, w.seq_lens, w.scale, table)
            pws = torch.empty(max(binding.hg_attn_partial_workspace_size(pdesc, packed), 256), dtype=torch.uint8, device=dev)

            def paged_step():
                hg.hg_attn_partial(w.q, kp, vp, w.seq_lens, packed, w.scale, m=m, l=l, o=o, workspace=pws, desc=pdesc)
                hg.hg_attn_merge(m, l, o, w.group_ptr, out=out, lse=lse)

            pms, _ = _time_steps(paged_step, max(steps // 4, 1), max(warmup // 4, 1), torch)
            paged["block_%d" % bt] = {"us": pms * 1e3, "gbps": w.kv_bytes / (pms * 1e-3) / 1e9}
            del kp, vp, table, pdesc, pkeep

        route_results = {
            "post_qk_route": {
                "offloaded_fraction": 0.8,
                "top_k": top_k,
                "logits_us": pq_logits_ms * 1e3,
                "select_us": pq_select_ms * 1e3,
                "select_resident_merge_us": pq_rest_ms * 1e3,
                "us": (pq_logits_ms + pq_rest_ms) * 1e3,
                "topk_us": pq_topk_ms * 1e3,  # hg_attn_topk: logits + selection in one call
                "one_call_us": pq_fused_ms * 1e3,  # hg_attn_topk + resident partial + merge
            },
            "pre_qk_route": {
                "offloaded_fraction": 0.8,
                "listed_tokens": top_k,
                "gather_us": pre_gather_ms * 1e3,
                "us": pre_step_ms * 1e3,
            },
            "paged_cache": paged,
            "concat_route": {
                "logits_us": logits_ms * 1e3,
                "concat_us": concat_ms * 1e3,
                "us": (logits_ms + concat_ms) * 1e3,
                "gbps": kv_bytes / ((logits_ms + concat_ms) * 1e-3) / 1e9,
                "logits_bytes": int(Hq) * int(ltok) * 4,
            },
        }
    res = {
        "workload": spec.name,
        "batch": spec.batch,
        "n_q_heads": spec.n_q_heads,
        "n_kv_heads": spec.n_kv_heads,
        "head_dim": spec.head_dim,
        "kv_dtype": spec.dtype,
        "tokens_total": int(w.seq_lens.sum()),
        "partitions": R,
        "span_tokens": span_tokens,
        "workgroups": n_workgroups,
        "kv_bytes": kv_bytes,
        "us_per_layer": ms * 1e3,
        "gbps": kv_bytes / (ms * 1e-3) / 1e9,
        "frac_hbm_peak": kv_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "full_path_us": full_ms * 1e3,
        "full_path_gbps": kv_bytes / (full_ms * 1e-3) / 1e9,
        "stream_kernel_us": kernel_ms * 1e3,
        "stream_kernel_gbps": kv_bytes / (kernel_ms * 1e-3) / 1e9,
        "host_wall_us_per_step": wall_ms * 1e3,
        "graph_replay_us": graph_ms * 1e3,
    }
    res.update(route_results)

    cpu = None
    if with_cpu_baseline:
        import numpy as np

        import oracle

        qn, kn, vn = (t.cpu().numpy() for t in (w.q, w.k, w.v))
        threads = oracle.max_threads()
        step()
        torch.cuda.synchronize()
        gpu_out = out.cpu().numpy()
        t0 = time.perf_counter()
        mo, lo, oo = oracle.attn_partial(qn, kn, vn, w.seq_lens, w.scale, w.ranges)
        ref, _ = oracle.attn_merge(mo, lo, oo, w.group_ptr)
        secs = time.perf_counter() - t0
        t1 = time.perf_counter()
        fref, _ = oracle.attn_full(qn, kn, vn, w.seq_lens, w.scale)
        fsecs = time.perf_counter() - t1
        err = float(np.abs(gpu_out - ref).max())
        cpu = {
            "value": kv_bytes / secs / 1e9,
            "unit": "GB/s",
            "cores": threads,
            "kind": "oracle",
            "sample": "whole workload %s: partial + merge once (%.2f s), then the unsplit definition once (%.2f s); fp64, "
                      "OpenMP over (range, head); about %.0f core-seconds in all" % (spec.name, secs, fsecs, (secs + fsecs) * threads),
            "seconds": secs,
            "unsplit_seconds": fsecs,
            "gpu_max_abs_err_vs_oracle": err,
            "oracle_split_vs_unsplit_max_abs": float(np.abs(ref - fref).max()),
        }
    del keep
    return res, cpu


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=1, help="index into workloads.ALL_WORKLOADS (headline: 1; 0-4 are the benchmark configurations, 5+ further shapes)")
    ap.add_argument("--others", type=str, default="0,2,3,4", help="comma list of further workloads to time ('' for none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-routes", action="store_true",
                    help="time the step and the unsplit path only (skips the concat, Post-QK^T, Pre-QK^T and paged-cache timings)")
    ap.add_argument("--span-tokens", type=int, default=0, help="force the span length (tuning)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run the library's plain 1 GiB device copy three times (known traffic: the "
                         "yardstick profiler byte counters are scaled by)")
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

    if args.calibration_copy:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            hg.hg_attn_calibration_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    head, cpu = run_workload(args.workload, args.steps, args.warmup, not args.no_cpu_baseline, torch, hg, W, not args.no_routes)
    others = []
    for tok in [t for t in args.others.split(",") if t.strip()]:
        i = int(tok)
        if i == args.workload:
            continue
        # (no empty_cache() between workloads: 288 GB hold every workload's tensors at once.  The
        # long workloads run for seconds at full HBM rate; their loops have been seen 4-5 % slower
        # for stretches of about a second whatever the order of the loops, so the figures of the
        # later workloads carry that much noise.)
        k = max(args.steps // 2, 5)
        r, _ = run_workload(i, k, max(args.warmup // 2, 2), False, torch, hg, W, not args.no_routes, loops=2)
        r["steps"] = k
        others.append(r)

    if head["kv_dtype"] != "f32" and head["n_q_heads"] // head["n_kv_heads"] >= 2:  # the library's own dispatch rule
        kernel_name = "hg_partial_gqa_kernel" if head["head_dim"] == 128 else "hg_partial_gqa64_kernel"
    else:
        kernel_name = "hg_partial_kernel"
    traffic, traffic_src = _profiled_traffic(kernel_name, head["workload"])
    line = {
        "metric": "decode attention effective KV GB/s (% of HBM peak) and us/layer at 1 GPU",
        "value": head["gbps"],
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["us_per_layer"] / 1e3,
        "us_per_layer": head["us_per_layer"],
        "graph_replay_us": head["graph_replay_us"],
        "frac_hbm_peak": head["frac_hbm_peak"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",  # fp16 K/V/q storage, fp32 products, sums and exponentials
        "data": "synthetic",
        "config": {k: head[k] for k in ("workload", "batch", "n_q_heads", "n_kv_heads", "head_dim", "kv_dtype",
                                        "tokens_total", "partitions", "span_tokens", "workgroups", "kv_bytes")},
        "roofline": {
            "bound": "hbm",
            "kernel": kernel_name,
            "achieved": head["stream_kernel_gbps"],
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": head["stream_kernel_gbps"] / HBM_PEAK_GBS,
            "traffic": traffic,
            "traffic_source": traffic_src,
            "kernel_us": head["stream_kernel_us"],
            "algorithmic_bytes_per_launch": head["kv_bytes"],
        },
        "cpu_baseline": cpu,
        "full_path": {"us": head["full_path_us"], "gbps": head["full_path_gbps"]},
        "concat_route": head.get("concat_route"),
        "post_qk_route": head.get("post_qk_route"),
        "pre_qk_route": head.get("pre_qk_route"),
        "paged_cache": head.get("paged_cache"),
        "other_workloads": others,
        "paper_context": PAPER_CONTEXT,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()

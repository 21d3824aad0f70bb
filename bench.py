#!/usr/bin/env python3
"""Benchmark of the tree-verification step on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input: ancestor sets,
tree-masked attention (with its split merge), vocabulary argmax, greedy acceptance and KV
compaction, enqueued through the C ABI (cb_verify_tree_device + cb_compact_kv).  The workload is
the 7B-shaped configuration (batch 1, 32 heads, head_dim 128, bf16, prefix 2048, 64-node tree from
the LRU drafter, logits [64, 32000]); inputs are resident in HBM before the timed region.  Steps
rotate over enough independent copies of (q, cache, logits) that every pass reads its K/V from HBM
rather than from the 256 MB last-level cache (--warm keeps one copy instead).

The steps are captured into a HIP graph (one graph holds one step per input copy) and the graph is
replayed; --no-graph launches them one by one from Python instead.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4000)
    ap.add_argument("--warmup", type=int, default=400)
    ap.add_argument("--config", type=int, default=2, help="workload 1..5 (default: the 7B-shaped one)")
    ap.add_argument("--copies", type=int, default=0, help="independent input copies to rotate over (0 = about 768 MB worth)")
    ap.add_argument("--warm", action="store_true", help="one input copy (cache-resident) instead of rotating copies")
    ap.add_argument("--layout", type=int, default=0, help="0 token-major cache, 1 head-major")
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--impl", type=int, default=0)
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--prefix", type=int, default=0, metavar="S",
                    help="override the workload's cached prefix length (a scaling probe, not the headline workload)")
    ap.add_argument("--layers", type=int, default=0, metavar="L",
                    help="instead of the headline: one step of an L-layer model -- tree attention on L distinct caches, "
                         "one logits scan + acceptance, one compaction of all L layers -- captured as one HIP graph")
    ap.add_argument("--decode-loop", type=int, default=0, metavar="STEPS",
                    help="instead of the headline: a closed decode loop (native drafter -> verify -> compact -> table "
                         "update) of STEPS steps on the 7B shape with a stand-in target; prints its own JSON line")
    ap.add_argument("--stage-probe", type=int, default=0, metavar="N",
                    help="for rocprofv3 --pmc runs: N launches of the attention stage alone on cold inputs, nothing else")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="for rocprofv3 --pmc runs: 50 attention launches, then one 256 MiB device copy as the calibration kernel")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2511_21699_amd import binding as B
    from paper_2511_21699_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.decode_loop:
        from paper_2511_21699_amd import decode_loop
        print(json.dumps(decode_loop.run(steps=args.decode_loop, warmup=2000, **({"prompt_len": args.prefix} if args.prefix else {}))))
        return
    case = W.make_config(args.config, **({"S": args.prefix} if args.prefix else {}))
    attn_bytes = case.attention_bytes()
    per_copy = attn_bytes + case.logits_bytes()
    copies = 1 if args.warm else (args.copies or max(2, -(-768 * 2 ** 20 // per_copy)))
    copies = max(1, min(copies, int(160e9 // per_copy)))
    if args.layers:
        copies = 1                       # the layers' distinct caches are the rotating inputs
    dcs = [B.DeviceCase(case, layout=args.layout) for _ in range(copies)]
    ver = B.Verifier(B.config_for_case(case, max_splits=72 if args.config == 4 else 0))
    if args.splits:
        ver.set_option("splits", args.splits)
    if args.impl:
        ver.set_option("attn_impl", args.impl)
    d_par = torch.from_numpy(case.parent).cuda()
    d_tok = torch.from_numpy(case.tokens).cuda()
    outs = [torch.empty_like(dc.q) for dc in dcs]
    d_len = torch.zeros(case.B, dtype=torch.int32, device="cuda")
    d_acc = torch.zeros(case.B, case.max_depth + 1, dtype=torch.int32, device="cuda")
    side = torch.cuda.Stream()          # a non-default stream: needed for graph capture, used for everything

    def bound_calls(with_compact):
        return [ver.bind_step(dc.q, dc.kv, case.kv_len, case.node_offsets, d_par, d_tok, dc.logits, outs[i], d_len, d_acc,
                              [dc.kv] if with_compact else [], stream=side) for i, dc in enumerate(dcs)]

    def make_runner(with_compact):
        """Returns (run(n_groups), steps_per_group): one group = one step on every input copy."""
        calls = bound_calls(with_compact)
        if len(calls) == 1:
            calls = calls * 20          # --warm: the same buffers 20 times per graph, so replay overhead stays small
        if args.no_graph:
            def run(n):
                for _ in range(n):
                    for c in calls:
                        c()
            return run, len(calls), "launches"
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            for c in calls[:2]:
                c()
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                for c in calls:
                    c()

        def run(n):
            with torch.cuda.stream(side):
                for _ in range(n):
                    graph.replay()
        return run, len(calls), "hipGraph"

    if args.layers:
        nl = args.layers
        base = dcs[0]
        ks = [base.k] + [torch.randn_like(base.k) * (case.D ** -0.5) for _ in range(nl - 1)]
        vs = [base.v] + [torch.randn_like(base.v) * (case.D ** -0.5) for _ in range(nl - 1)]
        qs = [base.q] + [torch.randn_like(base.q) for _ in range(nl - 1)]
        layer_outs = [torch.empty_like(base.q) for _ in range(nl)]
        paged = case.block_size > 0
        kvs = [B.kv_layer(k, v, base.block_table, layout=args.layout, paged=paged) for k, v in zip(ks, vs)]
        step = ver.bind_model_step(qs, kvs, case.kv_len, case.node_offsets, d_par, d_tok, base.logits, layer_outs,
                                   d_len, d_acc, stream=side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            step()
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                step()
            for _ in range(max(1, args.warmup // 10)):
                graph.replay()
            side.synchronize()
            n = max(1, args.steps // 10)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(side)
            for _ in range(n):
                graph.replay()
            e1.record(side)
            e1.synchronize()
        ms = e0.elapsed_time(e1) / n
        total_bytes = nl * attn_bytes + case.logits_bytes()
        print(json.dumps({"model_step": True, "layers": nl, "steps": n, "ms_per_step": round(ms, 4),
                          "steps_per_s": round(1e3 / ms, 1), "us_per_layer": round(ms * 1e3 / nl, 2),
                          "algorithmic_gbps": round(total_bytes / ms / 1e6, 1),
                          "pct_hbm_peak": round(100 * total_bytes / ms / 1e6 / HBM_PEAK_GBPS, 2),
                          "workload": f"configs[{args.config - 1}] {case.name} x {nl} layers, distinct caches ({nl * attn_bytes / 1e9:.2f} GB per step)",
                          "launch": "hipGraph", "accepted_len": d_len.cpu().tolist()[:4]}))
        return

    if args.stage_probe:
        ver.set_option("stages", 3)
        bound_calls(False)[0]()            # ancestor sets in place (scalar path)
        ver.set_option("stages", 2)
        calls = bound_calls(False)
        for i in range(args.stage_probe):
            calls[i % copies]()
            side.synchronize()
        print(json.dumps({"stage_probe": True, "attention_launches": args.stage_probe, "config": args.config}))
        return

    if args.traffic_probe:
        # 50 launches of the step's dominant kernel: the one-launch verification where the library
        # uses it, else the attention kernel alone
        bound_calls(False)[0]()
        side.synchronize()
        if not ver.last_launch_info()["fused"]:
            ver.set_option("stages", 3)
            bound_calls(False)[0]()
            ver.set_option("stages", 2)
        calls = bound_calls(False)
        for i in range(50):
            calls[i % copies]()
        side.synchronize()
        a = torch.empty(256 * 2 ** 20, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": True, "launches": 50, "fused": ver.last_launch_info()["fused"],
                          "copy_bytes_each_way": a.numel()}))
        return

    # ---- whole step: W warm-up steps, then exactly K timed steps
    run, per_group, how = make_runner(True)
    groups_w = max(1, args.warmup // per_group)
    groups = max(1, args.steps // per_group)
    steps, warmup = groups * per_group, groups_w * per_group
    run(groups_w)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(groups)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    accepted = d_len.cpu().tolist()
    info = ver.last_launch_info()

    # ---- one stage alone (attention incl. its split merge; argmax), HIP events on the launch stream
    def timed_stage(mask):
        ver.set_option("stages", 3)
        bound_calls(False)[0]()            # ancestor sets in place for the stage runs
        side.synchronize()
        ver.set_option("stages", mask)
        srun, spg, _ = make_runner(False)
        ver.set_option("stages", 15)
        srun(max(1, 100 // spg))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        n = max(1, args.steps // spg)
        e0.record(side)
        srun(n)
        e1.record(side)
        e1.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (n * spg)      # microseconds per launch

    attn_us = timed_stage(2)
    argmax_us = timed_stage(4)
    verify_us = timed_stage(15)          # attention + argmax + acceptance (no compaction): one launch when fused
    attn_gbps = attn_bytes / attn_us / 1e3

    # ---- what this machine delivers for a bare streaming read of as many bytes as the attention
    # sweeps: one launch of the library's read probe per cold buffer, replayed the same way
    def timed_stream_read():
        nb = (attn_bytes + 15) // 16 * 16
        bufs = [torch.randint(0, 2 ** 31 - 1, (nb // 4,), dtype=torch.int32, device="cuda") for _ in range(copies)]
        sink = torch.zeros(256, dtype=torch.int32, device="cuda")
        reps = 20 if copies == 1 else 1
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            B.probe_stream_read(bufs[0], nb, sink, stream=side)
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                for _ in range(reps):
                    for b in bufs:
                        B.probe_stream_read(b, nb, sink, stream=side)
            for _ in range(3):
                graph.replay()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            n = max(1, args.steps // (reps * copies))
            side.synchronize()
            e0.record(side)
            for _ in range(n):
                graph.replay()
            e1.record(side)
            e1.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (n * reps * copies)

    stream_us = timed_stream_read()
    stream_gbps = attn_bytes / stream_us / 1e3
    # The dominant kernel of the timed step.  Small calls run the whole verification as one launch
    # (k_verify_mfma): its algorithmic bytes are the attention's plus the logits'.  Otherwise it is
    # the attention kernel (with its split merge).
    if info["fused"]:
        roof_kernel = "cb::k_verify_mfma (tree attention incl. split merge + logits argmax + acceptance, one launch)"
        roof_bytes, roof_us = attn_bytes + case.logits_bytes(), verify_us
    else:
        roof_kernel = "cb::k_attn_mfma (tree attention incl. split merge)" if info["impl"] == 2 else "cb::k_attn_simt + cb::k_merge"
        roof_bytes, roof_us = attn_bytes, attn_us
    roof_gbps = roof_bytes / roof_us / 1e3

    out = {
        "metric": "tree-verify attention HBM GB/s (% of peak) + verify steps/s, 7B shape",
        "value": round(1e3 / ms_per_step, 1),
        "unit": "verify steps/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if case.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"configs[{args.config - 1}] {case.name}: B={case.B} Hq={case.Hq} Hkv={case.Hkv} D={case.D} "
                               f"prefix={case.kv_len.tolist() if case.B <= 4 else 'ragged'} nodes={case.total_nodes} V={case.V}",
                   "cache": "paged16" if case.block_size else "contiguous",
                   "layout": "token-major" if args.layout == 0 else "head-major",
                   "input_copies": copies, "cold_cache": not args.warm, "launch": how,
                   "accepted_len": accepted[:4]},
        "attention_us": round(attn_us, 3),
        "attention_gbps": round(attn_gbps, 1),
        "attention_pct_hbm_peak": round(100 * attn_gbps / HBM_PEAK_GBPS, 2),
        "stream_read": {"what": "one launch of a bare read kernel over as many bytes, same cold rotation and replay",
                        "us": round(stream_us, 3), "gbps": round(stream_gbps, 1),
                        "attention_pct_of_it": round(100 * attn_gbps / stream_gbps, 1)},
        "argmax_us": round(argmax_us, 3),
        "verify_us": round(verify_us, 3),
        "one_launch_verify": info["fused"],
        "splits": info["nsplit"],
        "roofline": {"bound": "hbm", "achieved": round(roof_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(roof_gbps / HBM_PEAK_GBPS, 4), "traffic": None,
                     "kernel": roof_kernel, "algorithmic_bytes": roof_bytes, "launch_us": round(roof_us, 3)},
    }
    traffic_file = os.path.join(ROOT, "profiles", "dominant_kernel_traffic.json")
    if os.path.exists(traffic_file):
        try:
            out["roofline"]["traffic"] = json.load(open(traffic_file)).get(f"config{args.config}")
        except Exception:
            pass

    # ---- the oracle on the host cores, same workload (a baseline beside the GPU number, not the target)
    if not args.no_cpu_baseline:
        from oracle import cb_oracle as O
        threads = min(O.num_threads(), os.cpu_count() or 1)
        all_rows = O.all_rows(case)
        rows, sample = all_rows, "whole workload"
        est = case.attention_flops() / 4 / 1.5e9 / max(threads, 1)      # rough seconds, ~1.5 G multiply-adds/s/core
        if est > 20:
            keep = max(threads, int(len(all_rows) * 20 / est))
            rows = all_rows[np.linspace(0, len(all_rows) - 1, keep).astype(int)]
            sample = f"attention: {keep} of {len(all_rows)} rows evenly spaced, time scaled up; argmax, acceptance, compaction: whole"
        t0 = time.perf_counter()
        O.attention_rows(case, rows, threads=threads)
        t_attn = (time.perf_counter() - t0) * (len(all_rows) / len(rows))
        t0 = time.perf_counter()
        a, res = O.verify(case)
        t_verify = time.perf_counter() - t0
        k2, v2 = case.k.copy(), case.v.copy()
        t0 = time.perf_counter()
        for b, (L, path, toks) in enumerate(res):
            O.compact(case, k2, v2, b, path)
        t_compact = time.perf_counter() - t0
        total = t_attn + t_verify + t_compact
        out["cpu_baseline"] = {"value": round(1.0 / total, 3), "unit": "verify steps/s", "cores": threads, "kind": "oracle",
                               "sample": sample, "attention_s": round(t_attn, 4), "argmax_accept_s": round(t_verify, 4),
                               "compact_s": round(t_compact, 5)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()

#!/usr/bin/env python3
"""Benchmark of the tree-verification step on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input: ancestor sets,
tree-masked attention (with its split merge), vocabulary argmax, greedy acceptance and KV
compaction, enqueued through the C ABI (cb_verify_tree_device + cb_compact_kv).  The headline
workload is the 7B-shaped configuration (batch 1, 32 heads, head_dim 128, bf16, prefix 2048,
64-node tree from the LRU drafter, logits [64, 32000]); inputs are resident in HBM before the
timed region.  Steps rotate over enough independent copies of (q, cache, logits) that every pass
reads its K/V from HBM rather than from the 256 MB last-level cache.

Steps are captured into HIP graphs and the graphs are replayed (--no-graph launches them one by one
from Python instead).  The timed region holds exactly --steps steps after --warmup untimed ones.
The per-stage figures (attention alone, argmax, the verification without the compaction) and the
`per_config` table over all five workloads do not depend on --steps: each is the median over
replays of at least 200 launches after at least 20 warm-up launches, timed with HIP events on the
launch stream.  Prints one JSON line.
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
MFMA_BF16_PEAK_TFLOPS = 2500.0
MIN_LAUNCHES, MIN_WARM = 200, 20


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4000)
    ap.add_argument("--warmup", type=int, default=400)
    ap.add_argument("--config", type=int, default=2, help="headline workload 1..5 (default: the 7B-shaped one)")
    ap.add_argument("--copies", type=int, default=0, help="independent input copies to rotate over (0 = about 768 MB worth)")
    ap.add_argument("--warm", action="store_true", help="headline on one input copy (cache-resident) instead of rotating copies")
    ap.add_argument("--layout", type=int, default=0, help="0 token-major cache, 1 head-major")
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--impl", type=int, default=0)
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true", help="skip the table over all five workloads")
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
                    help="for rocprofv3 --pmc runs: 50 launches of the step's dominant kernel, then one 256 MiB device copy as the calibration kernel")
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
        print(json.dumps(decode_loop.run(steps=args.decode_loop, warmup=400, **({"prompt_len": args.prefix} if args.prefix else {}))))
        return
    side = torch.cuda.Stream()          # a non-default stream: needed for graph capture, used for everything

    def timed_replays(run_once, launches_per_replay):
        """Median microseconds per launch over replays: >= MIN_WARM warm-up launches, then >= MIN_LAUNCHES timed
        ones, every replay bracketed by its own pair of HIP events on the launch stream."""
        warm = max(1, -(-MIN_WARM // launches_per_replay))
        reps = max(5, -(-MIN_LAUNCHES // launches_per_replay))
        with torch.cuda.stream(side):
            for _ in range(warm):
                run_once()
            side.synchronize()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
            for e0, e1 in evs:
                e0.record(side)
                run_once()
                e1.record(side)
            side.synchronize()
        per = sorted(e0.elapsed_time(e1) * 1e3 / launches_per_replay for e0, e1 in evs)
        return per[len(per) // 2], reps * launches_per_replay

    class Bench:
        """One workload on the device: input copies, a context, and graph builders."""

        def __init__(self, k, prefix=0, copies=0, warm=False):
            self.k = k
            self.case = case = W.make_config(k, **({"S": prefix} if prefix else {}))
            self.attn_bytes = case.attention_bytes()
            per_copy = self.attn_bytes + case.logits_bytes()
            n = 1 if warm else (copies or max(2, -(-768 * 2 ** 20 // per_copy)))
            self.copies = max(1, min(n, int(160e9 // per_copy)))
            self.dcs = [B.DeviceCase(case, layout=args.layout) for _ in range(self.copies)]
            self.ver = B.Verifier(B.config_for_case(case, max_splits=72 if k == 4 else 0))
            if args.splits:
                self.ver.set_option("splits", args.splits)
            if args.impl:
                self.ver.set_option("attn_impl", args.impl)
            self.d_par = torch.from_numpy(case.parent).cuda()
            self.d_tok = torch.from_numpy(case.tokens).cuda()
            self.outs = [torch.empty_like(dc.q) for dc in self.dcs]
            self.d_len = torch.zeros(case.B, dtype=torch.int32, device="cuda")
            self.d_acc = torch.zeros(case.B, case.max_depth + 1, dtype=torch.int32, device="cuda")

        def calls(self, with_compact, only=None):
            idx = range(self.copies) if only is None else only
            return [self.ver.bind_step(self.dcs[i].q, self.dcs[i].kv, self.case.kv_len, self.case.node_offsets, self.d_par,
                                       self.d_tok, self.dcs[i].logits, self.outs[i], self.d_len, self.d_acc,
                                       [self.dcs[i].kv] if with_compact else [], stream=side) for i in idx]

        def runner(self, calls):
            """A zero-argument function that enqueues `calls` once (as one HIP graph unless --no-graph)."""
            if args.no_graph:
                def run():
                    for c in calls:
                        c()
                return run
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                calls[0]()
                side.synchronize()
                with torch.cuda.graph(graph, stream=side):
                    for c in calls:
                        c()
            return graph.replay

        def stage_us(self, mask, copies=None):
            """Microseconds per launch of the stages in `mask` alone (2 attention incl. its merge, 4 argmax,
            15 the whole verification without the compaction), cold rotation over the input copies."""
            self.ver.set_option("stages", 3)
            self.calls(False, [0])[0]()            # ancestor sets in place for the scalar path's stage runs
            side.synchronize()
            self.ver.set_option("stages", mask)
            idx = list(range(self.copies)) if copies is None else copies
            calls = self.calls(False, idx)
            if len(calls) < 20 and self.attn_bytes < 64 * 2 ** 20:
                calls = calls * (-(-20 // len(calls)))    # small kernels: enough launches per replay to hide the replay's own cost
            run = self.runner(calls)
            self.ver.set_option("stages", 15)
            return timed_replays(run, len(calls))

        def close(self):
            self.ver.close()
            del self.dcs, self.outs
            torch.cuda.empty_cache()

    def table_row(bn):
        """One workload's stage figures (a row of `per_config`)."""
        case = bn.case
        attn_us, n_attn = bn.stage_us(2)
        argmax_us, _ = bn.stage_us(4)
        verify_us, _ = bn.stage_us(15)
        step_us, _ = timed_replays(bn.runner(bn.calls(True) * (1 if bn.attn_bytes >= 64 * 2 ** 20 else -(-20 // bn.copies))),
                                   bn.copies * (1 if bn.attn_bytes >= 64 * 2 ** 20 else -(-20 // bn.copies)))
        info = bn.ver.last_launch_info()
        gbps = bn.attn_bytes / attn_us / 1e3
        row = {"config": bn.k, "workload": case.name, "attention_us": round(attn_us, 2), "attention_gbps": round(gbps, 1),
               "frac_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4),
               "attention_tflops": round(case.attention_flops() / attn_us / 1e6, 1),
               "argmax_us": round(argmax_us, 2), "verify_us": round(verify_us, 2), "step_us": round(step_us, 2),
               "steps_per_s": round(1e6 / step_us, 1), "splits": info["nsplit"], "merge": info["merge"],
               "kernels_per_verification": info["kernels"], "one_launch_verify": info["fused"],
               "input_copies": bn.copies, "timed_launches_per_stage": n_attn,
               "attention_bytes": bn.attn_bytes, "attention_flops": case.attention_flops()}
        if bn.k in (3, 5):          # near the MFMA / HBM balance point: the matrix-core fraction beside the bandwidth
            row["frac_mfma_bf16_peak"] = round(case.attention_flops() / attn_us / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4)
        return row, dict(attn_us=attn_us, argmax_us=argmax_us, verify_us=verify_us, info=info)

    bn = Bench(args.config, prefix=args.prefix, copies=args.copies, warm=args.warm)
    case, ver, copies, attn_bytes = bn.case, bn.ver, bn.copies, bn.attn_bytes

    if args.layers:
        nl = args.layers
        base = bn.dcs[0]
        ks = [base.k] + [torch.randn_like(base.k) * (case.D ** -0.5) for _ in range(nl - 1)]
        vs = [base.v] + [torch.randn_like(base.v) * (case.D ** -0.5) for _ in range(nl - 1)]
        qs = [base.q] + [torch.randn_like(base.q) for _ in range(nl - 1)]
        layer_outs = [torch.empty_like(base.q) for _ in range(nl)]
        paged = case.block_size > 0
        kvs = [B.kv_layer(k, v, base.block_table, layout=args.layout, paged=paged) for k, v in zip(ks, vs)]
        step = ver.bind_model_step(qs, kvs, case.kv_len, case.node_offsets, bn.d_par, bn.d_tok, base.logits, layer_outs,
                                   bn.d_len, bn.d_acc, stream=side)
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
                          "launch": "hipGraph", "accepted_len": bn.d_len.cpu().tolist()[:4]}))
        return

    if args.stage_probe:
        ver.set_option("stages", 3)
        bn.calls(False, [0])[0]()            # ancestor sets in place (scalar path)
        ver.set_option("stages", 2)
        calls = bn.calls(False)
        for i in range(args.stage_probe):
            calls[i % copies]()
            side.synchronize()
        print(json.dumps({"stage_probe": True, "attention_launches": args.stage_probe, "config": args.config}))
        return

    if args.traffic_probe:
        # 50 launches of the step's dominant kernel: the one-launch verification where the library
        # uses it, else the attention kernel alone
        bn.calls(False, [0])[0]()
        side.synchronize()
        if not ver.last_launch_info()["fused"]:
            ver.set_option("stages", 3)
            bn.calls(False, [0])[0]()
            ver.set_option("stages", 2)
        calls = bn.calls(False)
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

    # ---- whole step: exactly W warm-up steps, then exactly K timed steps.  One graph holds one step per
    # input copy; a shorter graph holds the remainder, so the step counts are the ones asked for.
    def step_runners(n_steps):
        full, rest = divmod(n_steps, copies)
        runs = []
        if full:
            runs.append((bn.runner(bn.calls(True)), full))
        if rest:
            runs.append((bn.runner(bn.calls(True, list(range(rest)))), 1))
        return runs

    def play(runs):
        with torch.cuda.stream(side):
            for run, n in runs:
                for _ in range(n):
                    run()

    warm_runs, timed_runs = step_runners(args.warmup), step_runners(args.steps)
    play(warm_runs)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    play(timed_runs)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / max(1, args.steps)
    accepted = bn.d_len.cpu().tolist()

    # ---- one stage alone (attention incl. its split merge; argmax; the verification without the compaction)
    row, raw = table_row(bn)
    attn_us, argmax_us, verify_us, info = raw["attn_us"], raw["argmax_us"], raw["verify_us"], raw["info"]
    attn_gbps = attn_bytes / attn_us / 1e3
    warm_us, _ = bn.stage_us(2, copies=[0])           # one buffer, cache-resident: NOT the headline

    # ---- what this machine delivers for a bare streaming read of as many bytes as the attention
    # sweeps: one launch of the library's read kernel per cold buffer, replayed the same way
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
        return timed_replays(graph.replay, reps * copies)[0]

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
        "steps": args.steps,
        "warmup": args.warmup,
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
                   "input_copies": copies, "cold_cache": not args.warm,
                   "launch": "launches" if args.no_graph else "hipGraph",
                   "steps_per_graph": copies, "graph_replays_timed": [n for _, n in timed_runs],
                   "accepted_len": accepted[:4]},
        "attention_us": round(attn_us, 3),
        "attention_gbps": round(attn_gbps, 1),
        "attention_pct_hbm_peak": round(100 * attn_gbps / HBM_PEAK_GBPS, 2),
        "attention_us_warm_single_buffer": round(warm_us, 3),
        "stream_read": {"what": "one launch of a bare read kernel over as many bytes, same cold rotation and replay",
                        "us": round(stream_us, 3), "gbps": round(stream_gbps, 1),
                        "attention_pct_of_it": round(100 * attn_gbps / stream_gbps, 1)},
        "argmax_us": round(argmax_us, 3),
        "verify_us": round(verify_us, 3),
        "one_launch_verify": info["fused"],
        "splits": info["nsplit"],
        "merge": info["merge"],
        "stage_timing": f"median over replays, {row['timed_launches_per_stage']} timed launches after >= {MIN_WARM} warm-up launches, HIP events on the launch stream",
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

        def timed_attention(nthreads, budget_s):
            est = case.attention_flops() / 4 / 1.5e9 / max(nthreads, 1)      # rough seconds, ~1.5 G multiply-adds/s/core
            rows, sample = all_rows, "whole workload"
            if est > budget_s:
                keep = max(nthreads, int(len(all_rows) * budget_s / est))
                rows = all_rows[np.linspace(0, len(all_rows) - 1, keep).astype(int)]
                sample = f"attention: {keep} of {len(all_rows)} rows evenly spaced, time scaled up"
            t0 = time.perf_counter()
            O.attention_rows(case, rows, threads=nthreads)
            return (time.perf_counter() - t0) * (len(all_rows) / len(rows)), sample

        t_attn, sample = timed_attention(threads, 20)
        t0 = time.perf_counter()
        a, res = O.verify(case)
        t_verify = time.perf_counter() - t0
        k2, v2 = case.k.copy(), case.v.copy()
        t0 = time.perf_counter()
        for b, (L, path, toks) in enumerate(res):
            O.compact(case, k2, v2, b, path)
        t_compact = time.perf_counter() - t0
        total = t_attn + t_verify + t_compact
        t_attn1, sample1 = timed_attention(1, 8)
        total1 = t_attn1 + t_verify + t_compact
        out["cpu_baseline"] = {"value": round(1.0 / total, 3), "unit": "verify steps/s", "cores": threads, "kind": "oracle",
                               "sample": sample + "; argmax, acceptance, compaction: whole", "attention_s": round(t_attn, 4),
                               "argmax_accept_s": round(t_verify, 4), "compact_s": round(t_compact, 5),
                               "single_thread": {"value": round(1.0 / total1, 3), "unit": "verify steps/s", "cores": 1,
                                                 "sample": sample1 + "; argmax, acceptance, compaction: whole (as run above)",
                                                 "attention_s": round(t_attn1, 4)}}

    # ---- all five workloads, one after the other (each generated once; the headline's row is reused)
    if not args.no_per_config:
        rows = []
        bn.close()
        for k in range(1, 6):
            if k == args.config and not args.prefix and not args.warm:
                rows.append(row)
                continue
            b2 = Bench(k)
            rows.append(table_row(b2)[0])
            b2.close()
        out["per_config"] = rows
    print(json.dumps(out))


if __name__ == "__main__":
    main()

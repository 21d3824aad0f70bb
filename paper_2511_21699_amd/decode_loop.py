"""Closed Cacheback decode loop on one GPU, without a language model.

Every step of the paper's Section 3.2 runs for real -- the host drafter grows a tree from its LRU
table, the GPU verifies it (tree attention, argmax, greedy acceptance), the accepted K/V is
compacted, the table is updated over the new tokens by a sliding window -- except the model
forward that would produce q/k/v and the logits.  A stand-in target takes its place:

  * the "text the model would write" is a fixed synthetic token stream (truncated Zipf with copied
    spans, the recipe of the benchmark workloads); at a tree node whose root path spells the
    stream's continuation the target generates the stream's next token, at any other node a hash of
    the node (such nodes can never be accepted, their output is irrelevant);
  * logits are a fixed noise matrix in [-1, 1) with the generated token planted at 8.0 per node row;
  * q and the K/V cache hold fixed random numbers (the attention runs at its real shape and cost,
    its output is not consumed).

Because verification is lossless (Section 2.2), the emitted tokens must equal the stream
token for token whatever the drafter proposes; `run()` checks that after every step.

Two ways of keeping the accepted tokens' K/V (`policy`):
  * "compact": this library's -- cb_compact_kv moves the accepted nodes' K/V into place, the next
    tree's only non-cached token is its root;
  * "refeed": the paper's (Section 3.2: the tokens accepted in the last step are not KV-cached, they
    are fed again and count towards the total draft length) -- no compaction; the next tree starts
    with a chain of the tokens emitted last step, the draft subtree hangs under the chain's end, and
    the chain's K/V lands in its final slots by itself.

    python -m paper_2511_21699_amd.decode_loop --steps 1000          # one JSON line
"""
from __future__ import annotations

import argparse
import json
import time

import numpy as np

from . import binding as B
from . import drafter as PY
from . import workloads as W


def target_outputs(stream: np.ndarray, pos_root: int, parent, token, depth, vocab: int) -> np.ndarray:
    """Token the stand-in target generates at every tree node (see the module text)."""
    n = len(parent)
    on = np.zeros(n, dtype=bool)
    out = np.empty(n, dtype=np.int32)
    for i in range(n):
        on[i] = True if i == 0 else bool(on[parent[i]] and token[i] == stream[pos_root + depth[i]])
        if on[i]:
            out[i] = stream[pos_root + depth[i] + 1]
        else:
            out[i] = (int(token[i]) * 2654435761 + 40503 * int(depth[i]) + 977 * i) % vocab
    return out


def run(steps: int = 200, drafter: str = "native", node_budget: int = 64, depth_cap: int = 6, prompt_len: int = 2048,
        Hq: int = 32, Hkv: int = 32, D: int = 128, vocab: int = 32000, ll: int = 2, fl: int = 3, lc: int = 8192,
        fc: int = 4, seed: int = 7, device: str = "cuda:0", check_with=None, warmup: int = 50,
        policy: str = "compact", tables: str = "dynamic", corpus_tokens: int = 200000, use_only: str = "") -> dict:
    """Runs `warmup` untimed and then `steps` timed decode steps; returns timings and acceptance statistics.

    ``tables``: "dynamic" drafts from the dynamic table on the benchmark's stream; "dual" and "frozen" use a
    text with a shared phrase book and a frozen table built from a corpus sample of ``corpus_tokens`` tokens
    (Sections 3.3 and 4); ``use_only="dynamic"`` with ``tables="dual"`` is the same text without the frozen
    table (the "No Frozen" row of the paper's Table 1).
    ``check_with(step, parent, token, logits_rows, accepted_tokens)`` is an optional callback for tests
    (the step's tree, its logits rows on the device and everything the verification returned)."""
    import torch
    rng = np.random.default_rng(seed)
    room = (steps + warmup + 4) * (depth_cap + 1)
    if tables not in ("dynamic", "dual", "frozen"):
        raise ValueError("tables must be 'dynamic', 'dual' or 'frozen'")
    if tables == "dynamic":
        stream = W.zipf_stream(rng, prompt_len + room + 64, vocab)
        corpus = None
    else:
        # a "language" (phrase book), a corpus sample written in it for the frozen table (Section 4)
        # and, independently, the text to decode
        book = W.phrase_book(rng, 4000, vocab)
        corpus = W.phrase_stream(rng, corpus_tokens, vocab, book)
        stream = W.phrase_stream(rng, prompt_len + room + 64, vocab, book)
    gen = torch.Generator(device="cpu").manual_seed(seed)
    cap = prompt_len + room + node_budget
    dev = torch.device(device)
    k = (torch.randn(1, cap, Hkv, D, generator=gen) / D ** 0.5).to(torch.bfloat16).to(dev)
    v = (torch.randn(1, cap, Hkv, D, generator=gen) / D ** 0.5).to(torch.bfloat16).to(dev)
    q = torch.randn(node_budget, Hq, D, generator=gen).to(torch.bfloat16).to(dev)
    base = (torch.rand(node_budget, vocab, generator=gen) * 2 - 1).to(torch.bfloat16).to(dev)
    logits = base.clone()
    if policy not in ("compact", "refeed"):
        raise ValueError("policy must be 'compact' or 'refeed'")
    refeed = policy == "refeed"
    # with re-feeding the tree is a chain of up to depth_cap + 1 emitted tokens with the draft subtree below it
    cfg = B.make_config(Hq, Hkv, D, "bf16", "bf16", 1, node_budget, 2 * depth_cap + 1 if refeed else depth_cap, vocab)
    ver = B.Verifier(cfg, device=device)
    kv = B.kv_layer(k, v)
    # the step's C calls marshalled once: per-call conversions would cost as much as the GPU work (Section 1:
    # drafting takes microseconds, so the step should be bound by the GPU)
    attn_out = torch.empty_like(q)
    rows = torch.arange(node_budget, device=dev)
    frozen = None
    if drafter == "native":
        table = B.DraftTable(ll, fl, lc, fc)
        if corpus is not None:
            frozen = B.DraftTable(ll, fl, lc, fc, frozen_from=corpus)
        use = {"dynamic": [table], "dual": [table, frozen], "frozen": [frozen]}[use_only or tables]   # dynamic first (Section 3.3)
        growers = {}

        def grow(text, n, budget=node_budget):
            if budget not in growers:
                growers[budget] = B.TreeGrower(use, budget, depth_cap)
            return growers[budget].grow(text, n)
        update = lambda toks, start: table.update(toks, start)
    elif drafter == "python":
        if tables != "dynamic":
            raise ValueError("the frozen-table configurations use the native drafter")
        table = PY.CacheTable(ll, fl, lc, fc)
        grow = lambda text, n, budget=node_budget: PY.grow_tree(text[:n], [table], budget, depth_cap)
        update = lambda toks, start: table.update_sliding_window(toks, start)
    else:
        raise ValueError("drafter must be 'native' or 'python'")
    share = drafter == "native" and not refeed                      # the grower's output arrays are the call's tree arrays
    if share:
        growers[node_budget] = B.TreeGrower(use, node_budget, depth_cap)
        hs = ver.bind_host_step(q, kv, logits, attn_out, batch=1, layers=[kv], parent=growers[node_budget].parent,
                                tokens=growers[node_budget].token)
    else:
        hs = ver.bind_host_step(q, kv, logits, attn_out, batch=1, layers=[kv])
    emitted = np.empty(prompt_len + room + 8, dtype=np.int32)       # the whole text so far, prompt included
    emitted[:prompt_len] = stream[:prompt_len]
    n_text = prompt_len
    update(emitted[:n_text], 0)                                     # prompt initialisation (Section 3.3)
    t_draft = t_target = t_verify = t_compact = t_update = 0.0
    nodes_total, text0, kv_total = 0, prompt_len, 0
    pending = 1                                                     # tokens at the end of the text without cached K/V
    torch.cuda.synchronize(dev)
    wall0 = time.perf_counter()
    try:
        for step in range(-warmup, steps):
            if step == 0:                                           # the timed part starts here
                torch.cuda.synchronize(dev)
                t_draft = t_target = t_verify = t_compact = t_update = 0.0
                nodes_total, text0, kv_total = 0, n_text, 0
                wall0 = time.perf_counter()
            t0 = time.perf_counter()
            if refeed:
                # chain of the `pending` non-cached tokens, then the draft subtree under its last node;
                # the chain counts towards the budget (the paper's TDL counts non-cached tokens)
                sp, stk, sd = grow(emitted, n_text, node_budget - (pending - 1))
                c = pending - 1
                parent = np.concatenate([np.arange(-1, c - 1, dtype=np.int32), np.asarray(sp, dtype=np.int32) + c])
                parent[c] = c - 1
                token = np.concatenate([emitted[n_text - pending:n_text - 1], np.asarray(stk, dtype=np.int32)])
                depth = np.concatenate([np.arange(c, dtype=np.int32), np.asarray(sd, dtype=np.int32) + c])
            else:
                parent, token, depth = grow(emitted, n_text)
            t1 = time.perf_counter()
            parent = np.asarray(parent, dtype=np.int32)
            token = np.asarray(token, dtype=np.int32)
            n = len(parent)
            root_pos = n_text - pending                              # text index of tree node 0
            # ---- stand-in for the model forward: logits rows for the tree's nodes
            outs = target_outputs(stream, root_pos, parent, token, depth, vocab)
            logits[:n].copy_(base[:n])
            logits[rows[:n], torch.from_numpy(outs).to(dev).long()] = 8.0
            torch.cuda.synchronize(dev)                            # (so that the stand-in's GPU time is not booked on the verification)
            t2 = time.perf_counter()
            hs.kv_len[0] = root_pos
            hs.node_offsets[1] = n
            if not share:
                hs.parent[:n] = parent
                hs.tokens[:n] = token
            hs.verify()
            acc_len, acc_tok = hs.accepted_len, hs.accepted_tokens
            t3 = time.perf_counter()
            if not refeed:
                hs.compact()
            t4 = time.perf_counter()
            L = int(acc_len[0]) - (pending - 1)                      # newly accepted draft tokens
            if L < 0:
                raise AssertionError(f"step {step}: the re-fed chain itself was not accepted")
            new = acc_tok[0, pending - 1:pending + L]
            if check_with is not None:
                check_with(step + warmup, parent, token, logits[:n], acc_tok[0, :int(acc_len[0]) + 1])
            if not np.array_equal(new, stream[n_text:n_text + L + 1]):
                raise AssertionError(f"step {step}: emitted {new.tolist()} but the text continues "
                                     f"{stream[n_text:n_text + L + 1].tolist()} (verification must be lossless)")
            emitted[n_text:n_text + L + 1] = new
            old = n_text
            n_text += L + 1
            pending = L + 1 if refeed else 1
            t5 = time.perf_counter()
            update(emitted[:n_text], old - (fl - 1))               # every window that touches a new token
            t6 = time.perf_counter()
            t_draft += t1 - t0; t_target += t2 - t1; t_verify += t3 - t2; t_compact += t4 - t3; t_update += t6 - t5
            nodes_total += n
            kv_total += root_pos
        torch.cuda.synchronize(dev)
        wall = time.perf_counter() - wall0
    finally:
        ver.close()
        if drafter == "native":
            table.close()
            if frozen is not None:
                frozen.close()
    us = lambda t: round(t / steps * 1e6, 2)
    own = t_draft + t_verify + t_compact + t_update                 # everything except the stand-in target
    return {"steps": steps, "drafter": drafter, "policy": policy, "tables": tables, "warmup": warmup, "tokens_emitted": int(n_text - text0),
            "mean_accepted_tokens_per_step": round((n_text - text0) / steps, 3),
            "mean_tree_nodes": round(nodes_total / steps, 1), "mean_kv_len": round(kv_total / steps, 1),
            "draft_us": us(t_draft), "verify_us": us(t_verify), "compact_us": us(t_compact), "table_update_us": us(t_update),
            "stand_in_target_us": us(t_target),
            "steps_per_s_without_target": round(steps / own, 1), "steps_per_s_wall": round(steps / wall, 1),
            "lossless": True,
            "shape": f"Hq={Hq} Hkv={Hkv} D={D} V={vocab} prompt={prompt_len} TDL={node_budget} depth<={depth_cap} "
                     f"LL={ll} FL={fl} LC={lc} FC={fc}"}


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--drafter", default="native", choices=["native", "python"])
    ap.add_argument("--prompt", type=int, default=2048)
    ap.add_argument("--nodes", type=int, default=64)
    ap.add_argument("--policy", default="compact", choices=["compact", "refeed"])
    ap.add_argument("--tables", default="dynamic", choices=["dynamic", "dual", "frozen"],
                    help="dynamic table only (on the benchmark's stream), or the paper's table configurations on a "
                         "text with a shared phrase book: dual (dynamic then frozen), frozen only")
    ap.add_argument("--ablate", action="store_true", help="the three table configurations of the paper's Table 1 on one text")
    ap.add_argument("--warmup", type=int, default=400,
                    help="untimed steps first; the text keeps growing through them (about 2.2 tokens a step), so with the "
                         "default prompt of 2048 the 1000 timed steps see prefixes of about 3000 to 5200 tokens, 4100 on "
                         "average (the output's mean_kv_len): the 7B benchmark shape")
    args = ap.parse_args()
    if args.ablate:
        for name, kw in (("Dual", dict(tables="dual")), ("No Frozen", dict(tables="dual", use_only="dynamic")),
                         ("Only Frozen", dict(tables="frozen"))):
            r = run(steps=args.steps, prompt_len=args.prompt, node_budget=args.nodes, warmup=min(args.warmup, 200), **kw)
            print(json.dumps({"configuration": name, "mean_accepted_tokens_per_step": r["mean_accepted_tokens_per_step"],
                              "mean_tree_nodes": r["mean_tree_nodes"], "draft_us": r["draft_us"],
                              "steps_per_s_without_target": r["steps_per_s_without_target"]}))
        return
    print(json.dumps(run(steps=args.steps, drafter=args.drafter, prompt_len=args.prompt, node_budget=args.nodes,
                         warmup=args.warmup, policy=args.policy, tables=args.tables)))


if __name__ == "__main__":
    main()

"""Independent re-statements used to pin the oracle (numpy / pure Python, float64).

None of this goes through ``oracle/``: it is the textbook side of each pin.
"""
from __future__ import annotations

import numpy as np

from paper_2511_21699_amd import workloads as W


def slot_rows(case, which: str, seq: int, slots, head: int) -> np.ndarray:
    """float64 [len(slots), D] rows of K or V for one sequence / kv head, through the cache layout."""
    arr = case.k if which == "k" else case.v
    out = np.empty((len(slots), case.D), dtype=np.float64)
    for t, s in enumerate(slots):
        if case.block_size > 0:
            blk = int(case.block_table[seq, s // case.block_size])
            row = arr[blk, s % case.block_size, head]
        else:
            row = arr[seq, s, head]
        out[t] = W.to_f64(row, case.dtype)
    return out


def causal_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float) -> np.ndarray:
    """Textbook causal attention of one head: q, k, v are [T, D]; row t sees keys 0..t."""
    T = q.shape[0]
    s = (q @ k.T) * scale
    mask = np.tril(np.ones((T, T), dtype=bool))
    s = np.where(mask, s, -np.inf)
    s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    p /= p.sum(axis=1, keepdims=True)
    return p @ v


def root_to_leaf_paths(parent):
    n = len(parent)
    has_child = [False] * n
    for i in range(1, n):
        has_child[parent[i]] = True
    paths = []
    for leaf in range(n):
        if has_child[leaf]:
            continue
        p = []
        x = leaf
        while x >= 0:
            p.append(x)
            x = int(parent[x])
        paths.append(p[::-1])
    return paths


def per_path_attention(case, scale=None):
    """Tree attention by brute force: every root-to-leaf path is run as an ordinary causal
    sequence [prefix..., path nodes] on its own.  Returns float64 [sum_nodes, Hq, D] and asserts
    that paths sharing a node agree on it."""
    if scale is None:
        scale = 1.0 / np.sqrt(case.D)
    total = int(case.node_offsets[-1])
    out = np.full((total, case.Hq, case.D), np.nan)
    g = case.Hq // case.Hkv
    qf = W.to_f64(case.q, case.dtype)
    for b in range(case.B):
        lo, hi = int(case.node_offsets[b]), int(case.node_offsets[b + 1])
        S = int(case.kv_len[b])
        par = case.parent[lo:hi]
        for path in root_to_leaf_paths(par):
            slots = list(range(S)) + [S + a for a in path]
            for h in range(case.Hq):
                k = slot_rows(case, "k", b, slots, h // g)
                v = slot_rows(case, "v", b, slots, h // g)
                # queries for the prefix positions are irrelevant to the path rows: use zeros
                q = np.zeros((len(slots), case.D))
                for j, a in enumerate(path):
                    q[S + j] = qf[lo + a, h]
                o = causal_attention(q, k, v, scale)
                for j, a in enumerate(path):
                    row = o[S + j]
                    if not np.isnan(out[lo + a, h, 0]):
                        np.testing.assert_allclose(out[lo + a, h], row, rtol=1e-12, atol=1e-14)
                    out[lo + a, h] = row
    assert not np.isnan(out).any()
    return out


def sequential_greedy_accept(parent, tokens, a):
    """Walk every root-to-leaf path token by token: a draft token is accepted when it equals what
    the model generated at the previous accepted node.  Longest walk wins; ties go to the walk
    whose last accepted node has the lowest index.  Returns (L, path, emitted tokens)."""
    best_path = [0]
    for path in root_to_leaf_paths(parent):
        walked = [0]
        for node in path[1:]:
            if tokens[node] != a[walked[-1]]:
                break
            walked.append(node)
        if len(walked) > len(best_path) or (len(walked) == len(best_path) and walked[-1] < best_path[-1]):
            best_path = walked
    emitted = [int(a[x]) for x in best_path]
    return len(best_path) - 1, best_path, emitted

"""Seeded synthetic inputs for the tree-verification path (numpy only, host side).

This module only *draws inputs*: query/key/value tensors, draft trees, draft tokens, logits and
(for the ragged case) a paged cache with a shuffled block table.  It holds none of the
verification arithmetic (no attention, no acceptance, no compaction); both the CPU oracle and the
HIP library are fed from here so that they see bit-identical inputs.

The five workloads stand in for what the paper measured on (SpecBench prompts decoded by Vicuna
models, Section 4 of the paper), which is not available offline: they keep the structure the paper
describes -- draft trees grown breadth-first from an LRU n-gram table (Sections 3.1-3.2), a node
budget of the order of the paper's total draft length (TDL = 96), per-edge acceptance around 0.5-0.6
(the paper's mean accepted tokens of 2.42, Table 1) -- with synthetic token streams and random
tensors in place of model activations.

bf16 tensors are carried as ``uint16`` bit patterns (numpy has no bfloat16).
"""
from __future__ import annotations

import os
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

from .drafter import CacheTable, grow_tree

BASE_SEED = 25112169900
BLOCK_TOKENS = 16


# ----------------------------------------------------------------------------- bf16 bit helpers
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact float64 view of a tensor stored as float32 or as bf16 bit patterns."""
    if dtype == "bf16":
        return bf16_bits_to_f32(a).astype(np.float64)
    return np.asarray(a, dtype=np.float32).astype(np.float64)


_SLAB = 1 << 23


def _normal(rng: np.random.Generator, shape, dtype: str, scale: float = 1.0) -> np.ndarray:
    """N(0, scale^2) drawn in float32, rounded (RNE) to bf16 when asked.

    Small tensors come straight from ``rng``.  Large ones are cut into fixed slabs, each drawn from
    its own generator keyed by (one 63-bit draw from ``rng``, slab index), so the result does not
    depend on how many threads fill the slabs."""
    n = int(np.prod(shape))
    if n <= _SLAB:
        x = rng.standard_normal(n, dtype=np.float32)
        if scale != 1.0:
            x *= np.float32(scale)
        return (x if dtype == "f32" else f32_to_bf16_bits(x)).reshape(shape)
    key = int(rng.integers(0, 2 ** 63 - 1))
    out = np.empty(n, dtype=np.float32 if dtype == "f32" else np.uint16)

    def fill(s: int) -> None:
        e = min(n, s + _SLAB)
        g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([key, s // _SLAB])))
        x = g.standard_normal(e - s, dtype=np.float32)
        if scale != 1.0:
            x *= np.float32(scale)
        out[s:e] = x if dtype == "f32" else f32_to_bf16_bits(x)

    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
        list(ex.map(fill, range(0, n, _SLAB)))
    return out.reshape(shape)


# ----------------------------------------------------------------------------- case container
@dataclass
class VerifyCase:
    """One batch of verification inputs.  Layouts (innermost dimension contiguous):

    q        [sum_nodes, Hq, D]
    k, v     contiguous cache: [B, capacity, Hkv, D];  paged: [num_blocks, block_size, Hkv, D]
    logits   [sum_nodes, V]
    Cache slot ``kv_len[b] + i`` of sequence b holds the K/V of its tree node i.
    """
    name: str
    dtype: str                 # "f32" | "bf16" for q/k/v and logits alike
    B: int
    Hq: int
    Hkv: int
    D: int
    V: int
    max_depth: int
    block_size: int            # 0 = contiguous
    kv_len: np.ndarray         # int32 [B]
    node_offsets: np.ndarray   # int32 [B+1]
    parent: np.ndarray         # int32 [sum_nodes], local index, -1 at each root
    tokens: np.ndarray         # int32 [sum_nodes]
    q: np.ndarray
    k: np.ndarray
    v: np.ndarray
    logits: np.ndarray
    block_table: Optional[np.ndarray] = None   # int32 [B, max_blocks] when paged
    info: Dict = field(default_factory=dict)

    @property
    def total_nodes(self) -> int:
        return int(self.node_offsets[-1])

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def attention_bytes(self) -> int:
        """Algorithmic bytes of the attention: prefix and tree K/V once, Q in, O out."""
        b = self.elem_bytes
        n = np.diff(self.node_offsets).astype(np.int64)
        kv = int(((self.kv_len.astype(np.int64) + n) * self.Hkv * self.D * b * 2).sum())
        qo = int(n.sum()) * self.Hq * self.D * b * 2
        return kv + qo

    def attention_flops(self) -> int:
        n = np.diff(self.node_offsets).astype(np.int64)
        return int((4 * n * self.Hq * (self.kv_len.astype(np.int64) + n) * self.D).sum())

    def logits_bytes(self) -> int:
        return self.total_nodes * self.V * self.elem_bytes


# ----------------------------------------------------------------------------- trees
def random_tree(rng: np.random.Generator, n: int, max_children: int, max_depth: int,
                force_depth: bool) -> Tuple[np.ndarray, np.ndarray]:
    """Random parent array: each new node hangs under a uniformly chosen earlier node that still
    has fewer than ``max_children`` children and depth below ``max_depth``.  With ``force_depth``
    the draw is repeated until some node sits exactly at ``max_depth``."""
    if n < 1:
        raise ValueError("a tree has at least its root")
    while True:
        parent = np.full(n, -1, dtype=np.int32)
        depth = np.zeros(n, dtype=np.int32)
        nchild = np.zeros(n, dtype=np.int32)
        for i in range(1, n):
            ok = np.flatnonzero((nchild[:i] < max_children) & (depth[:i] < max_depth))
            if ok.size == 0:
                raise ValueError("tree budget does not fit under the branching/depth caps")
            p = int(ok[rng.integers(ok.size)])
            parent[i], depth[i] = p, depth[p] + 1
            nchild[p] += 1
        if not force_depth or n <= max_depth or depth.max() == max_depth:
            return parent, depth


def chain_tree(n: int) -> np.ndarray:
    return np.arange(-1, n - 1, dtype=np.int32)


def star_tree(n: int) -> np.ndarray:
    p = np.zeros(n, dtype=np.int32)
    p[0] = -1
    return p


def tree_depths(parent: np.ndarray) -> np.ndarray:
    d = np.zeros(len(parent), dtype=np.int32)
    for i in range(1, len(parent)):
        d[i] = d[parent[i]] + 1
    return d


# ----------------------------------------------------------------------------- token stream + drafter trees
def zipf_stream(rng: np.random.Generator, length: int, vocab: int, exponent: float = 1.1,
                p_repeat: float = 0.3, span: Tuple[int, int] = (4, 16)) -> np.ndarray:
    """Token stream with burstiness: at each decision point, with probability ``p_repeat`` copy an
    earlier span (length uniform in ``span``, start uniform), else emit one truncated-Zipf token
    (P(rank r) ~ r^-exponent over ``vocab`` ranks, id = r - 1, inverse-CDF sampling)."""
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-exponent)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    out = np.empty(length + span[1], dtype=np.int32)
    u = rng.random(length + 1)
    z = np.minimum(np.searchsorted(cdf, rng.random(length + 1)), vocab - 1).astype(np.int32)
    t = 0
    step = 0
    while t < length:
        if t >= span[0] and u[step] < p_repeat:
            ln = int(rng.integers(span[0], span[1] + 1))
            ln = min(ln, t)
            s = int(rng.integers(0, t - ln + 1))
            out[t:t + ln] = out[s:s + ln]
            t += ln
        else:
            out[t] = z[step]
            t += 1
        step += 1
    return out[:length].copy()


def phrase_book(rng: np.random.Generator, phrases: int, vocab: int, span: Tuple[int, int] = (3, 8),
                exponent: float = 1.1) -> list:
    """A fixed list of token phrases (lengths uniform in ``span``, tokens truncated-Zipf): the part of
    a synthetic "language" that every text written in it shares."""
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-exponent)
    cdf = np.cumsum(w) / w.sum()
    return [np.minimum(np.searchsorted(cdf, rng.random(int(rng.integers(span[0], span[1] + 1)))), vocab - 1).astype(np.int32)
            for _ in range(phrases)]


def phrase_stream(rng: np.random.Generator, length: int, vocab: int, book: list, p_phrase: float = 0.45,
                  p_repeat: float = 0.2, span: Tuple[int, int] = (4, 16), exponent: float = 1.1) -> np.ndarray:
    """Text in the "language" of ``book``: at each decision point a phrase of the book (Zipf-weighted
    choice) with probability ``p_phrase``, a copy of an earlier span of this text with probability
    ``p_repeat``, else one truncated-Zipf token.  Two texts over the same book share their phrases
    (what a table built offline from a corpus can know) but not their own repetitions (what only a
    table updated while decoding can know)."""
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-exponent)
    cdf = np.cumsum(w) / w.sum()
    bw = np.arange(1, len(book) + 1, dtype=np.float64) ** (-exponent)
    bcdf = np.cumsum(bw) / bw.sum()
    out = np.empty(length + 64, dtype=np.int32)
    t = 0
    while t < length:
        u = rng.random()
        if u < p_phrase:
            ph = book[min(int(np.searchsorted(bcdf, rng.random())), len(book) - 1)]
            out[t:t + len(ph)] = ph
            t += len(ph)
        elif u < p_phrase + p_repeat and t >= span[0]:
            ln = min(int(rng.integers(span[0], span[1] + 1)), t)
            s0 = int(rng.integers(0, t - ln + 1))
            out[t:t + ln] = out[s0:s0 + ln]
            t += ln
        else:
            out[t] = min(int(np.searchsorted(cdf, rng.random())), vocab - 1)
            t += 1
    return out[:length].copy()


def drafter_tree(rng: np.random.Generator, n_nodes: int, depth_cap: int, vocab: int = 32000,
                 stream_len: int = 32768, ll: int = 2, fl: int = 3, fc: int = 4, lc: int = 8192,
                 max_children: int = 4) -> Tuple[np.ndarray, np.ndarray, Dict]:
    """Draft tree of exactly ``n_nodes`` nodes from the LRU drafter run over a synthetic stream.

    The table is warmed by a sliding window over the stream up to a cut point (the last position
    whose LL-token leader already has two or more followers); the root is the token at the cut.
    If the drafter stops short of the budget (no leaf has a follower), the tree is padded
    deterministically -- the stand-in for the frozen-table growth of the paper's Section 3.3 --
    by hanging Zipf-drawn tokens under the lowest-index node with spare branching and depth.
    """
    stream = zipf_stream(rng, stream_len, vocab)
    probe = CacheTable(ll, fl, lc, fc)
    cut = -1
    for t in range(ll, stream_len - fl + 1):
        probe.insert(stream[t - ll:t].tolist(), stream[t:t + fl].tolist())
        # after this insert the table covers followers starting at <= t, i.e. tokens up to t+fl-1
        end = t + fl - 1
        if len(probe.peek(stream[end - ll + 1:end + 1].tolist())) >= 2:
            cut = end
    if cut < 0:
        cut = stream_len - 1
    table = CacheTable(ll, fl, lc, fc)
    context = stream[:cut + 1].tolist()
    table.update_sliding_window(context)
    parent, token, depth = grow_tree(context, [table], n_nodes, depth_cap)
    drafted = len(parent)
    # pad (frozen-table stand-in)
    nchild = [0] * len(parent)
    for i in range(1, len(parent)):
        nchild[parent[i]] += 1
    kids = [set() for _ in parent]
    for i in range(1, len(parent)):
        kids[parent[i]].add(token[i])
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-1.1)
    cdf = np.cumsum(w) / w.sum()
    host = 0
    while len(parent) < n_nodes:
        while host < len(parent) and not (nchild[host] < max_children and depth[host] < depth_cap):
            host += 1
        if host >= len(parent):
            raise ValueError("cannot pad the tree under the caps")
        while True:
            tk = int(min(np.searchsorted(cdf, rng.random()), vocab - 1))
            if tk not in kids[host]:
                break
        parent.append(host); token.append(tk); depth.append(depth[host] + 1)
        nchild.append(0); kids.append(set())
        nchild[host] += 1; kids[host].add(tk)
    info = {"drafted_nodes": drafted, "cut": cut, "table_leaders": len(table)}
    return np.asarray(parent, dtype=np.int32), np.asarray(token, dtype=np.int32), info


# ----------------------------------------------------------------------------- logits / tokens
def _row_max_plus_one(row: np.ndarray, dtype: str):
    if dtype == "bf16":
        m = float(bf16_bits_to_f32(row).max())
        return f32_to_bf16_bits(np.array([m + 1.0], dtype=np.float32))[0]
    return np.float32(row.max() + np.float32(1.0))


def plant_logits(rng: np.random.Generator, logits: np.ndarray, dtype: str, parent: np.ndarray,
                 tokens: np.ndarray, p: float) -> int:
    """For each internal node, with probability ``p``, pick one child uniformly and raise the
    logit of that child's token to (row maximum + 1), which makes it the row's unique maximum."""
    n = len(parent)
    kids: List[List[int]] = [[] for _ in range(n)]
    for i in range(1, n):
        kids[parent[i]].append(i)
    planted = 0
    for i in range(n):
        if kids[i] and rng.random() < p:
            c = kids[i][int(rng.integers(len(kids[i])))]
            logits[i, tokens[c]] = _row_max_plus_one(logits[i], dtype)
            planted += 1
    return planted


def tokens_from_row_maxima(rng: np.random.Generator, logits: np.ndarray, dtype: str,
                           parent: np.ndarray, vocab: int, p_match: float) -> np.ndarray:
    """Draft tokens for random trees: each non-root node copies, with probability ``p_match``, the
    index of the first maximum of its parent's logits row (a lookup used only to build inputs),
    otherwise a uniform token.  Siblings may repeat a token."""
    n = len(parent)
    vals = bf16_bits_to_f32(logits) if dtype == "bf16" else logits
    first_max = np.argmax(vals, axis=1).astype(np.int32)
    tok = rng.integers(0, vocab, size=n).astype(np.int32)
    hit = rng.random(n) < p_match
    for i in range(1, n):
        if hit[i]:
            tok[i] = first_max[parent[i]]
    return tok


# ----------------------------------------------------------------------------- cache builders
def _contiguous_cache(rng, B, cap, Hkv, D, dtype, scale):
    k = _normal(rng, (B, cap, Hkv, D), dtype, scale)
    v = _normal(rng, (B, cap, Hkv, D), dtype, scale)
    return k, v


def _paged_layout(rng, kv_len, n_nodes, block):
    need = [(int(s) + int(n) + block - 1) // block for s, n in zip(kv_len, n_nodes)]
    total = int(sum(need))
    perm = rng.permutation(total).astype(np.int32)
    table = np.full((len(need), max(need)), -1, dtype=np.int32)
    o = 0
    for b, nb in enumerate(need):
        table[b, :nb] = perm[o:o + nb]
        o += nb
    return table, total


# ----------------------------------------------------------------------------- the five workloads
_SPECS = {
    1: dict(name="tiny", dtype="f32", B=1, Hq=8, Hkv=8, D=64, V=1000, S=256, N=15, depth=4, branch=2,
            tree="random", p=0.6, kv_scale=1.0),
    2: dict(name="7b", dtype="bf16", B=1, Hq=32, Hkv=32, D=128, V=32000, S=2048, N=64, depth=6, branch=4,
            tree="drafter", p=0.6, kv_scale=128 ** -0.5),
    3: dict(name="gqa", dtype="bf16", B=1, Hq=32, Hkv=8, D=128, V=32000, S=8192, N=128, depth=8, branch=4,
            tree="drafter", p=0.5, kv_scale=128 ** -0.5),
    4: dict(name="ragged", dtype="bf16", B=16, Hq=32, Hkv=32, D=128, V=32000, S=(512, 16384), N=(32, 96),
            depth=8, branch=4, tree="drafter", p=0.6, kv_scale=128 ** -0.5, paged=True),
    5: dict(name="long13b", dtype="bf16", B=1, Hq=40, Hkv=40, D=128, V=128256, S=65536, N=256, depth=10,
            branch=4, tree="random", p=0.4, kv_scale=128 ** -0.5),
}


def config_spec(k: int) -> Dict:
    return dict(_SPECS[k])


def make_config(k: int, seed_offset: int = 0, peaked: bool = False, **override) -> VerifyCase:
    """Build workload ``k`` (1..5).  ``override`` may shrink S / N / V / B / Hq / Hkv (same recipe,
    smaller sizes) for cases the CPU oracle must finish in seconds.  ``peaked`` multiplies the
    queries by 4*sqrt(D) so that the softmax concentrates on few keys and outputs are O(1)."""
    sp = config_spec(k)
    sp.update(override)
    seed = BASE_SEED + 100 * k + seed_offset
    rng = np.random.Generator(np.random.PCG64(seed))
    dtype, B, Hq, Hkv, D, V = sp["dtype"], sp["B"], sp["Hq"], sp["Hkv"], sp["D"], sp["V"]
    # --- per-sequence sizes
    if isinstance(sp["S"], tuple):
        kv_len = rng.integers(sp["S"][0], sp["S"][1] + 1, size=B).astype(np.int32)
    else:
        kv_len = np.full(B, sp["S"], dtype=np.int32)
    if isinstance(sp["N"], tuple):
        n_nodes = rng.integers(sp["N"][0], sp["N"][1] + 1, size=B).astype(np.int32)
    else:
        n_nodes = np.full(B, sp["N"], dtype=np.int32)
    node_offsets = np.zeros(B + 1, dtype=np.int32)
    node_offsets[1:] = np.cumsum(n_nodes)
    total = int(node_offsets[-1])
    # --- trees (+ tokens for drafter trees)
    parents, toks, infos = [], [], []
    for b in range(B):
        n = int(n_nodes[b])
        if sp["tree"] == "random":
            par, _ = random_tree(rng, n, sp["branch"], sp["depth"], force_depth=(k == 1))
            parents.append(par); toks.append(None); infos.append({})
        else:
            sub = np.random.Generator(np.random.PCG64(seed * 1000 + 7 + b))
            par, tk, info = drafter_tree(sub, n, sp["depth"], vocab=V, stream_len=sp.get("stream_len", 32768),
                                         max_children=sp["branch"])
            parents.append(par); toks.append(tk); infos.append(info)
    parent = np.concatenate(parents).astype(np.int32)
    # --- tensors
    q = _normal(rng, (total, Hq, D), dtype, 1.0)
    if peaked:
        qf = to_f64(q, dtype) * (4.0 * np.sqrt(D))
        q = f32_to_bf16_bits(qf.astype(np.float32)) if dtype == "bf16" else qf.astype(np.float32)
    block_table = None
    if sp.get("paged"):
        block_table, nblocks = _paged_layout(rng, kv_len, n_nodes, BLOCK_TOKENS)
        kc = _normal(rng, (nblocks, BLOCK_TOKENS, Hkv, D), dtype, sp["kv_scale"])
        vc = _normal(rng, (nblocks, BLOCK_TOKENS, Hkv, D), dtype, sp["kv_scale"])
        block = BLOCK_TOKENS
    else:
        cap = int((kv_len + n_nodes).max())
        kc, vc = _contiguous_cache(rng, B, cap, Hkv, D, dtype, sp["kv_scale"])
        block = 0
    logits = _normal(rng, (total, V), dtype, 1.0)
    # --- draft tokens / planting
    tokens = np.empty(total, dtype=np.int32)
    planted = 0
    for b in range(B):
        lo, hi = int(node_offsets[b]), int(node_offsets[b + 1])
        if sp["tree"] == "random":
            tokens[lo:hi] = tokens_from_row_maxima(rng, logits[lo:hi], dtype, parents[b], V, sp["p"])
        else:
            tokens[lo:hi] = toks[b]
            planted += plant_logits(rng, logits[lo:hi], dtype, parents[b], toks[b], sp["p"])
    depth_max = max(int(tree_depths(p).max()) for p in parents)
    return VerifyCase(name=sp["name"], dtype=dtype, B=B, Hq=Hq, Hkv=Hkv, D=D, V=V, max_depth=max(sp["depth"], depth_max),
                      block_size=block, kv_len=kv_len, node_offsets=node_offsets, parent=parent, tokens=tokens,
                      q=q, k=kc, v=vc, logits=logits, block_table=block_table,
                      info={"seed": seed, "planted_rows": planted, "drafter": infos, "config": k,
                            "peaked": peaked})


def custom_case(seed: int, dtype: str, B: int, Hq: int, Hkv: int, D: int, V: int, kv_len, parents,
                paged: bool = False, kv_scale: float = 1.0, q_scale: float = 1.0, p_match: float = 0.6,
                extra_capacity: int = 0) -> VerifyCase:
    """Free-form case for edge tests: explicit prefix lengths and parent arrays."""
    rng = np.random.Generator(np.random.PCG64(seed))
    kv_len = np.asarray(kv_len, dtype=np.int32)
    n_nodes = np.asarray([len(p) for p in parents], dtype=np.int32)
    node_offsets = np.zeros(B + 1, dtype=np.int32)
    node_offsets[1:] = np.cumsum(n_nodes)
    total = int(node_offsets[-1])
    q = _normal(rng, (total, Hq, D), dtype, q_scale)
    block_table = None
    if paged:
        block_table, nblocks = _paged_layout(rng, kv_len, n_nodes, BLOCK_TOKENS)
        kc = _normal(rng, (nblocks, BLOCK_TOKENS, Hkv, D), dtype, kv_scale)
        vc = _normal(rng, (nblocks, BLOCK_TOKENS, Hkv, D), dtype, kv_scale)
        block = BLOCK_TOKENS
    else:
        cap = int((kv_len + n_nodes).max()) + extra_capacity
        kc, vc = _contiguous_cache(rng, B, cap, Hkv, D, dtype, kv_scale)
        block = 0
    logits = _normal(rng, (total, V), dtype, 1.0)
    tokens = np.empty(total, dtype=np.int32)
    for b in range(B):
        lo, hi = int(node_offsets[b]), int(node_offsets[b + 1])
        tokens[lo:hi] = tokens_from_row_maxima(rng, logits[lo:hi], dtype, np.asarray(parents[b]), V, p_match)
    parent = np.concatenate([np.asarray(p, dtype=np.int32) for p in parents])
    depth_max = max(int(tree_depths(np.asarray(p)).max()) for p in parents)
    return VerifyCase(name="custom", dtype=dtype, B=B, Hq=Hq, Hkv=Hkv, D=D, V=V, max_depth=max(depth_max, 1),
                      block_size=block, kv_len=kv_len, node_offsets=node_offsets, parent=parent, tokens=tokens,
                      q=q, k=kc, v=vc, logits=logits, block_table=block_table, info={"seed": seed})

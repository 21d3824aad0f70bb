"""The drafter oracle (oracle/drafter_oracle.py) against what the paper fixes, and the two product
drafters -- the native one behind cacheback_drafter.h and the Python one that builds the workloads
-- against the oracle, bit for bit."""
import ctypes as C
import json
import os
import re

import numpy as np
import pytest

from oracle.drafter_oracle import TableOracle, build_frozen_oracle, grow_tree_oracle
from paper_2511_21699_amd import binding as B
from paper_2511_21699_amd import drafter as P
from paper_2511_21699_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


# ----------------------------------------------------------------------------- pins of the oracle
def test_oracle_reproduces_the_figure_2_example():
    """Section 3.2 / Figure 2 caption: prefix 'At dawn the fox', LL = FL = 2, three followers of 'the fox'."""
    with open(os.path.join(GOLDEN, "fig2_example.json")) as f:
        g = json.load(f)
    voc = g["vocab"]
    t = TableOracle(g["LL"], g["FL"], 64, 8)
    leader = [voc[w] for w in g["first_query_leader"]]
    for fol in reversed(g["first_query_followers"]):
        t.insert(leader, [voc[w] for w in fol])
    assert t.query(leader, refresh=False) == [tuple(voc[w] for w in fol) for fol in g["first_query_followers"]]
    parent, token, depth = grow_tree_oracle([voc[w] for w in g["prefix"]], [t], 96, 8)
    assert parent == g["tree_parent"] and token == [voc[w] for w in g["tree_tokens"]]


def test_oracle_table_hand_traced_lru_in_both_domains():
    """Section 3.1: capacity LC = 2 leaders, FC = 2 followers; every state below is traced by hand."""
    t = TableOracle(1, 1, 2, 2)
    t.insert([1], [10]); t.insert([2], [20]); t.insert([1], [11])
    assert t.size() == (2, 3)
    t.insert([3], [30])                                   # leader 2 is the least recently inserted: evicted
    assert t.query([2], refresh=False) == [] and t.query([1], refresh=False) == [(11,), (10,)]
    t.insert([1], [10])                                   # present follower becomes the most recent
    assert t.query([1], refresh=False) == [(10,), (11,)]
    t.insert([1], [12])                                   # FC = 2: follower 11 is evicted
    assert t.query([1], refresh=False) == [(12,), (10,)]
    t.query([3])                                          # a lookup counts as a use of the leader ...
    t.insert([4], [40])                                   # ... so leader 1 goes, not leader 3
    assert t.query([1], refresh=False) == [] and t.query([3], refresh=False) == [(30,)]
    t.frozen = True
    t.insert([9], [9]); t.insert([3], [31])
    assert t.size() == (2, 2)


def test_oracle_sliding_window_enumerates_every_pair():
    """Section 3.2 (update) / 3.3 (prompt): every window of LL + FL consecutive tokens is one pair."""
    toks = [5, 6, 7, 8, 9, 10]
    t = TableOracle(2, 2, 100, 100)
    t.update(toks)
    assert t.size() == (3, 3)
    for i in range(2, 5):
        assert t.query(toks[i - 2:i], refresh=False) == [tuple(toks[i:i + 2])]
    t2 = TableOracle(2, 2, 100, 100)
    t2.update(toks, start=4)                              # only the window whose follower starts at index 4
    assert t2.size() == (1, 1) and t2.query([7, 8], refresh=False) == [(9, 10)]


def test_oracle_tree_growth_properties():
    """Section 3.2: breadth-first, TDL counts every token of the tree, followers cut at the budget;
    trees are valid (parent[i] < i, depths consistent), no two siblings carry the same token."""
    rng = np.random.default_rng(3)
    stream = W.zipf_stream(rng, 4000, 50)
    t = TableOracle(2, 3, 500, 4)
    t.update(stream[:3000])
    for cut in range(3000, 3040):
        for budget, cap, crt in ((1, 5, 0), (7, 2, 0), (40, 6, 0), (40, 6, 16)):
            parent, token, depth = grow_tree_oracle(stream[:cut], [t], budget, cap, crt)
            n = len(parent)
            assert 1 <= n <= budget and token[0] == stream[cut - 1] and parent[0] == -1
            assert all(0 <= parent[i] < i and depth[i] == depth[parent[i]] + 1 for i in range(1, n))
            assert max(depth) <= cap
            sib = {}
            for i in range(1, n):
                assert (parent[i], token[i]) not in sib
                sib[(parent[i], token[i])] = i
            # every root child chain spells a follower prefix of the root's leader
            fols = t.query(stream[cut - 2:cut], refresh=False)
            for i in range(1, n):
                if parent[i] == 0 and cap >= 1:
                    assert any(f[0] == token[i] for f in fols)


def test_oracle_chaining_reserve_holds_budget_back_for_later_rounds():
    t = TableOracle(1, 1, 64, 8)
    for f in (2, 3, 4, 5, 6):
        t.insert([1], [f])
    for leader in (2, 3, 4, 5, 6):
        t.insert([leader], [7])
    p0, _, d0 = grow_tree_oracle([1], [t], 6, 8, 0)          # the first round takes the whole budget
    assert d0 == [0, 1, 1, 1, 1, 1]
    p1, _, d1 = grow_tree_oracle([1], [t], 6, 8, 2)          # two tokens are kept for the second round
    assert d1 == [0, 1, 1, 1, 2, 2]


# ----------------------------------------------------------------------------- product drafters vs the oracle
def _random_ops(seed, ll, fl, lc, fc, vocab, n_ops):
    rng = np.random.default_rng(seed)
    for _ in range(n_ops):
        leader = rng.integers(0, vocab, ll).tolist()
        r = rng.random()
        if r < 0.35:
            yield "query", leader, None
        elif r < 0.40:
            yield "peek", leader, None
        else:
            yield "insert", leader, rng.integers(0, max(2, vocab // 2), fl).tolist()


@pytest.mark.parametrize("seed,ll,fl,lc,fc,vocab", [(0, 1, 2, 6, 3, 10), (1, 2, 3, 40, 4, 6), (2, 3, 1, 5, 1, 3), (3, 2, 2, 1, 2, 4)])
def test_native_and_python_tables_match_the_oracle(seed, ll, fl, lc, fc, vocab):
    o, n, p = TableOracle(ll, fl, lc, fc), B.DraftTable(ll, fl, lc, fc), P.CacheTable(ll, fl, lc, fc)
    for op, leader, fol in _random_ops(seed, ll, fl, lc, fc, vocab, 4000):
        if op == "insert":
            o.insert(leader, fol); n.insert(leader, fol); p.insert(leader, fol)
        else:
            refresh = op == "query"
            want = o.query(leader, refresh)
            assert n.query(leader, refresh) == want
            assert (p.query(leader) if refresh else p.peek(leader)) == want
        assert n.size() == o.size()
    n.freeze(); o.frozen = True
    n.insert([0] * ll, [0] * fl)
    assert n.size() == o.size()
    n.close()


@pytest.mark.parametrize("seed", range(4))
def test_native_and_python_tree_growth_match_the_oracle(seed):
    rng = np.random.default_rng(100 + seed)
    stream = W.zipf_stream(rng, 6000, 200 if seed % 2 else 30)
    ll, fl, lc, fc = [(2, 3, 300, 4), (1, 2, 50, 3), (3, 2, 2000, 2), (2, 4, 64, 8)][seed]
    tabs = [(TableOracle(ll, fl, lc, fc), B.DraftTable(ll, fl, lc, fc), P.CacheTable(ll, fl, lc, fc)),
            (TableOracle(ll, 2, 200, 2), B.DraftTable(ll, 2, 200, 2), P.CacheTable(ll, 2, 200, 2))]
    for o, n, p in tabs[1:]:                                   # the second table is a frozen one (Section 3.3)
        o.update(stream[:1500]); n.update(stream[:1500]); p.update_sliding_window(stream[:1500])
        o.frozen = True; n.freeze(); p.freeze()
    o, n, p = tabs[0]
    o.update(stream[:4000]); n.update(stream[:4000]); p.update_sliding_window(stream[:4000])
    pos = 4000
    for step in range(60):
        budget, cap, crt = int(rng.integers(1, 70)), int(rng.integers(0, 9)), int(rng.integers(0, 20))
        use = 2 if step % 3 == 0 else 1
        ctx = stream[:pos] if step % 7 else stream[pos - 1:pos]          # sometimes a context shorter than a leader
        want = grow_tree_oracle(ctx, [t[0] for t in tabs[:use]], budget, cap, crt)
        if step % 2:
            got_n = B.grow_tree(ctx, [t[1] for t in tabs[:use]], budget, cap, crt)
        else:                                                             # the pre-marshalled form the decode loop uses
            text = np.ascontiguousarray(ctx, dtype=np.int32)
            got_n = B.TreeGrower([t[1] for t in tabs[:use]], budget, cap, crt).grow(text, len(text))
        got_p = P.grow_tree(ctx, [t[2] for t in tabs[:use]], budget, cap, crt)
        for w, a, b in zip(want, got_n, got_p):
            assert list(a) == w and list(b) == w
        adv = int(rng.integers(1, 6))                                    # the decode loop's sliding-window update
        start = pos - (fl - 1)
        pos += adv
        o.update(stream[:pos], start); n.update(stream[:pos], start); p.update_sliding_window(stream[:pos], start)
        assert n.size() == o.size()
    for t3 in tabs:
        t3[1].close()


def test_drafter_header_symbols_are_exported_and_bad_arguments_are_refused():
    text = open(os.path.join(ROOT, "include", "cacheback_drafter.h")).read()
    names = sorted(set(re.findall(r"\b(cbd_[a-z_]+)\s*\(", text)))
    assert names == sorted(B.DRAFTER_EXPORTS)
    L = B.load()
    for name in names:
        assert hasattr(L, name)
    h = C.c_void_p()
    for bad in ((0, 1, 1, 1), (1, 0, 1, 1), (1, 1, 0, 1), (1, 1, 1, 0), (17, 1, 1, 1), (1, 1, 1, 65)):
        assert L.cbd_table_create(*bad, C.byref(h)) == B.CB_EINVAL
    t = B.DraftTable(2, 2, 4, 2)
    one = np.zeros(1, dtype=np.int32)
    n = C.c_int32(0)
    assert L.cbd_grow_tree((C.c_void_p * 1)(t.h), 1, B._ip(one), 0, 4, 4, 0, B._ip(one), B._ip(one), B._ip(one), C.byref(n)) == B.CB_EINVAL
    assert L.cbd_grow_tree((C.c_void_p * 1)(t.h), 1, B._ip(one), 1, 0, 4, 0, B._ip(one), B._ip(one), B._ip(one), C.byref(n)) == B.CB_EINVAL
    t.close()


def test_frozen_table_build_oracle_hand_counted():
    """Section 4: most frequent leaders, then each leader's most frequent followers (hand-counted sample)."""
    #        windows (LL = 1, FL = 1):  1>2 2>1 1>2 2>3 3>1 1>3 3>1 1>2   -> leader 1 x4, 2 x2, 3 x2
    toks = [1, 2, 1, 2, 3, 1, 3, 1, 2]
    t = build_frozen_oracle(toks, 1, 1, 2, 1)
    assert t.size() == (2, 2)                              # leaders 1 and 2 (2 and 3 tie at two; 2 came first)
    assert t.query([1], refresh=False) == [(2,)]           # after 1: 2 x3, 3 x1
    assert t.query([2], refresh=False) == [(1,)]           # after 2: 1 and 3 once each; 1 came first
    assert t.query([3], refresh=False) == []
    t.insert([9], [9])
    assert t.size() == (2, 2)                              # frozen
    t2 = build_frozen_oracle(toks, 1, 1, 8, 8)
    assert t2.query([1], refresh=False) == [(2,), (3,)] and t2.query([3], refresh=False) == [(1,)]


@pytest.mark.parametrize("seed,ll,fl,lc,fc,vocab", [(0, 2, 3, 50, 3, 12), (1, 1, 1, 5, 2, 6), (2, 3, 2, 1000, 4, 40)])
def test_native_frozen_table_build_matches_the_oracle(seed, ll, fl, lc, fc, vocab):
    rng = np.random.default_rng(300 + seed)
    toks = W.zipf_stream(rng, 3000, vocab)
    o = build_frozen_oracle(toks, ll, fl, lc, fc)
    n = B.DraftTable(ll, fl, lc, fc, frozen_from=toks)
    assert n.size() == o.size()
    for row in o.rows:
        assert n.query(row[0], refresh=False) == o.query(row[0], refresh=False)
    n.insert([0] * ll, [1] * fl)
    assert n.size() == o.size()
    n.close()

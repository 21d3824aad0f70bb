"""Host logic: the LRU n-gram drafter (paper Sections 3.1-3.3) and the synthetic workload recipes."""
import json
import os

import numpy as np
import pytest

from paper_2511_21699_amd import workloads as W
from paper_2511_21699_amd.drafter import CacheTable, grow_tree

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


class ListLRU:
    """Twenty-line list-based model of the table of Section 3.1 (front = least recent)."""

    def __init__(self, lc, fc):
        self.lc, self.fc, self.rows = lc, fc, []          # rows: [leader, [followers]]

    def _find(self, leader):
        for r in self.rows:
            if r[0] == leader:
                return r
        return None

    def query(self, leader):
        r = self._find(leader)
        if r is None:
            return []
        self.rows.remove(r); self.rows.append(r)
        return r[1][::-1]

    def insert(self, leader, fol):
        r = self._find(leader)
        if r is None:
            if len(self.rows) >= self.lc:
                self.rows.pop(0)
            self.rows.append([leader, [fol]])
            return
        self.rows.remove(r); self.rows.append(r)
        if fol in r[1]:
            r[1].remove(fol); r[1].append(fol)
        else:
            if len(r[1]) >= self.fc:
                r[1].pop(0)
            r[1].append(fol)


@pytest.mark.parametrize("seed", range(5))
def test_cache_table_matches_list_model_and_respects_capacities(seed):
    rng = np.random.default_rng(seed)
    t, m = CacheTable(1, 2, 6, 3), ListLRU(6, 3)
    for _ in range(2000):
        leader = (int(rng.integers(0, 10)),)
        if rng.random() < 0.4:
            assert t.query(leader) == m.query(leader)
        else:
            fol = (int(rng.integers(0, 3)), int(rng.integers(0, 3)))
            t.insert(leader, fol); m.insert(leader, fol)
        assert len(t) <= 6 and all(len(t.peek(r[0])) <= 3 for r in m.rows)
    assert [tuple(r[0]) for r in m.rows] == list(t._t.keys())


def test_query_refreshes_leader_but_not_followers():
    t = CacheTable(1, 1, 2, 2)
    t.insert((1,), (10,)); t.insert((2,), (20,))
    t.query((1,))                       # leader 1 becomes most recent
    t.insert((3,), (30,))               # evicts leader 2
    assert t.peek((2,)) == [] and t.peek((1,)) == [(10,)]
    t.insert((1,), (11,)); t.query((1,)); t.insert((1,), (12,))   # follower 10 is the LRU despite the query
    assert t.peek((1,)) == [(12,), (11,)]


def test_frozen_table_ignores_inserts():
    t = CacheTable(1, 1, 4, 4)
    t.insert((1,), (2,))
    t.freeze()
    t.insert((1,), (3,)); t.insert((5,), (6,))
    assert t.peek((1,)) == [(2,)] and t.peek((5,)) == []


def test_figure2_tree_growth():
    with open(os.path.join(GOLDEN, "fig2_example.json")) as f:
        g = json.load(f)
    voc = g["vocab"]
    t = CacheTable(g["LL"], g["FL"], 64, 8)
    leader = [voc[w] for w in g["first_query_leader"]]
    for fol in reversed(g["first_query_followers"]):       # inserted oldest-last so the query returns the paper's order
        t.insert(leader, [voc[w] for w in fol])
    assert t.peek(leader) == [tuple(voc[w] for w in fol) for fol in g["first_query_followers"]]
    parent, token, depth = grow_tree([voc[w] for w in g["prefix"]], [t], node_budget=96, depth_cap=8)
    assert parent == g["tree_parent"]
    assert token == [voc[w] for w in g["tree_tokens"]]


def test_tree_growth_is_breadth_first_budgeted_and_merges_prefixes():
    t = CacheTable(1, 2, 64, 8)
    t.insert((1,), (2, 3)); t.insert((1,), (2, 4)); t.insert((3,), (5, 6)); t.insert((4,), (7, 8))
    parent, token, depth = grow_tree([9, 1], [t], node_budget=96, depth_cap=8)
    assert token[:4] == [1, 2, 4, 3] and parent[:4] == [-1, 0, 1, 1]      # shared first token merged
    assert sorted(token[4:]) == [5, 6, 7, 8] and max(depth) == 4
    parent, token, depth = grow_tree([9, 1], [t], node_budget=5, depth_cap=8)
    assert len(parent) == 5                                               # TDL counts the root
    parent, token, depth = grow_tree([9, 1], [t], node_budget=96, depth_cap=3)
    assert max(depth) == 3
    frozen = CacheTable(1, 2, 64, 8); frozen.insert((6,), (1, 1)); frozen.freeze()
    p2, t2, d2 = grow_tree([9, 1], [t, frozen], node_budget=96, depth_cap=8)
    assert len(p2) == 10 and t2[-2:] == [1, 1]                            # frozen table grows the tree further


def test_sliding_window_update_captures_all_pairs():
    t = CacheTable(2, 2, 64, 8)
    t.update_sliding_window([1, 2, 3, 4, 5])
    assert t.peek((1, 2)) == [(3, 4)] and t.peek((2, 3)) == [(4, 5)] and len(t) == 2


@pytest.mark.parametrize("k", [1, 2])
def test_workload_recipes_are_seeded_and_well_formed(k):
    a, b = W.make_config(k), W.make_config(k)
    for f in ("q", "k", "v", "logits", "parent", "tokens", "kv_len"):
        assert np.array_equal(getattr(a, f), getattr(b, f))
    c = W.make_config(k, seed_offset=1)
    assert not np.array_equal(a.logits, c.logits)
    sp = W.config_spec(k)
    assert a.total_nodes == sp["N"] and a.parent[0] == -1 and (a.parent[1:] < np.arange(1, sp["N"])).all()
    d = W.tree_depths(a.parent)
    assert d.max() <= sp["depth"] and np.bincount(a.parent[1:]).max() <= sp["branch"]
    if k == 1:
        assert d.max() == 4 and a.q.dtype == np.float32
    else:
        assert a.q.dtype == np.uint16 and a.attention_bytes() == 35651584


def test_ragged_paged_layout_small():
    c = W.make_config(4, B=3, S=(20, 200), N=(5, 12), Hq=2, Hkv=2, V=100, stream_len=2000)
    assert c.block_size == 16 and c.block_table.shape[0] == 3
    used = c.block_table[c.block_table >= 0]
    assert len(np.unique(used)) == len(used) == c.k.shape[0]              # a permutation of the pool
    need = (c.kv_len + np.diff(c.node_offsets) + 15) // 16
    assert ((c.block_table >= 0).sum(axis=1) == need).all()


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 3.0e38], dtype=np.float32)
    b = W.f32_to_bf16_bits(x)
    # 1+2^-8 is a tie between 1.0 and 1+2^-7 -> even mantissa (1.0); 1+3*2^-8 ties up to 1+2^-6
    assert W.bf16_bits_to_f32(b).tolist()[:4] == [1.0, 1.0, 1.015625, -1.0]
    assert np.isfinite(W.bf16_bits_to_f32(b)[4])

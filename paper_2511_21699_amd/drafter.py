"""Host-side LRU n-gram drafter of Cacheback decoding (serial host code, never on the GPU).

Follows the paper's Section 3.1 (cache table: leaders -> followers, two LRU domains) and
Section 3.2 (breadth-first growth of the draft-token tree by recursive table queries, bounded by
the total draft length TDL and the chaining-reserved tokens CRT), plus Section 3.3 (a frozen
table queried after the dynamic one while the budget allows, prompt initialisation by a sliding
window).  It only *produces inputs* (trees) for the verification path; nothing here is used to
check results.

Readings where the paper is silent (they shape the workload, not the verified results):
  * a query returns followers most-recently-inserted first;
  * re-inserting a follower that is already present refreshes its recency (insertion is the only
    thing that does, Section 3.1);
  * followers are cut token by token at the node budget and at the depth cap;
  * followers sharing a prefix under the same leaf are merged trie-style;
  * CRT reserves budget for BFS rounds after the first one.
"""
from __future__ import annotations

from collections import OrderedDict
from typing import Iterable, List, Optional, Sequence, Tuple


class CacheTable:
    """Leader -> follower-list table with LRU eviction in both domains (Section 3.1).

    ``ll``/``fl`` are the leader/follower lengths in tokens, ``lc``/``fc`` the capacities.
    The paper's prototype uses Python's OrderedDict; so does this one.
    """

    def __init__(self, ll: int, fl: int, lc: int, fc: int, frozen: bool = False):
        if min(ll, fl, lc, fc) < 1:
            raise ValueError("LL, FL, LC, FC must all be >= 1")
        self.ll, self.fl, self.lc, self.fc = ll, fl, lc, fc
        self.frozen = frozen
        self._t: "OrderedDict[Tuple[int, ...], OrderedDict[Tuple[int, ...], None]]" = OrderedDict()

    def __len__(self) -> int:
        return len(self._t)

    def peek(self, leader: Sequence[int]) -> List[Tuple[int, ...]]:
        """Followers of ``leader`` (most recent first) without touching recency."""
        f = self._t.get(tuple(leader))
        return list(reversed(f)) if f is not None else []

    def query(self, leader: Sequence[int]) -> List[Tuple[int, ...]]:
        """Followers of ``leader``, most recent first; refreshes the leader's recency."""
        key = tuple(leader)
        f = self._t.get(key)
        if f is None:
            return []
        if not self.frozen:
            self._t.move_to_end(key)
        return list(reversed(f))

    def insert(self, leader: Sequence[int], follower: Sequence[int]) -> None:
        """Accept one leader-follower pair; a frozen table ignores it (Section 3.3)."""
        if self.frozen:
            return
        key, fol = tuple(leader), tuple(follower)
        if len(key) != self.ll or len(fol) != self.fl:
            raise ValueError("leader/follower length mismatch")
        f = self._t.get(key)
        if f is None:
            if len(self._t) >= self.lc:
                self._t.popitem(last=False)          # evict the LRU leader and its followers
            self._t[key] = OrderedDict([(fol, None)])
            return
        self._t.move_to_end(key)                      # inserting refreshes the leader
        if fol in f:
            f.move_to_end(fol)
        else:
            if len(f) >= self.fc:
                f.popitem(last=False)                 # evict this leader's LRU follower
            f[fol] = None

    def update_sliding_window(self, tokens: Sequence[int], start: int = 0) -> None:
        """Insert every (leader, follower) window whose follower starts at index >= ``start``.

        Used for the prompt initialisation (Section 3.3) and for the per-step update over the
        newly accepted tokens (Section 3.2): pass the whole sequence and the index of the first
        new token minus (FL - 1) so that all windows touching new tokens are captured.
        """
        ll, fl = self.ll, self.fl
        n = len(tokens)
        first = max(ll, start)
        for t in range(first, n - fl + 1):
            self.insert(tokens[t - ll:t], tokens[t:t + fl])

    def freeze(self) -> "CacheTable":
        self.frozen = True
        return self


def grow_tree(context: Sequence[int], tables: Iterable[CacheTable], node_budget: int,
              depth_cap: int, crt: int = 0) -> Tuple[List[int], List[int], List[int]]:
    """Grow a draft-token tree under the last token of ``context`` (Section 3.2).

    Node 0 is the root (the last, not yet KV-cached, token of the context).  Returns
    ``(parent, token, depth)`` with ``parent[0] == -1`` and ``parent[i] < i``.  ``node_budget``
    is TDL: it counts the root as well as the draft tokens.  ``tables`` are queried in order
    (dynamic first, then frozen, Section 3.3), each one growing the tree breadth-first from the
    current leaves until no leaf has a follower or the budget is reached.
    """
    if len(context) < 1:
        raise ValueError("context must hold at least the root token")
    parent, token, depth = [-1], [int(context[-1])], [0]
    children: List[dict] = [{}]

    def path_tokens(node: int, need: int) -> List[int]:
        out: List[int] = []
        while node >= 0 and len(out) < need:
            out.append(token[node])
            node = parent[node]
        out.reverse()
        if len(out) < need:                            # reach back into the context before the root
            extra = need - len(out)
            ctx = list(context[:-1])
            out = [int(x) for x in ctx[max(0, len(ctx) - extra):]] + out
        return out

    for table in tables:
        ll = table.ll
        leaves = [i for i in range(len(parent)) if not children[i]]
        first_round = True
        while leaves and len(parent) < node_budget:
            # CRT keeps part of the budget for the second and deeper BFS rounds.
            limit = node_budget - crt if (first_round and crt > 0) else node_budget
            limit = max(limit, min(node_budget, len(parent) + 1))
            new_leaves: List[int] = []
            for leaf in leaves:
                if len(parent) >= limit:
                    break
                key = path_tokens(leaf, ll)
                if len(key) < ll:
                    continue
                for fol in table.query(key):
                    node = leaf
                    for tk in fol:
                        if depth[node] >= depth_cap:
                            break
                        nxt = children[node].get(int(tk))
                        if nxt is None:
                            if len(parent) >= limit:
                                break
                            nxt = len(parent)
                            parent.append(node); token.append(int(tk)); depth.append(depth[node] + 1)
                            children.append({})
                            children[node][int(tk)] = nxt
                        node = nxt
                    if node != leaf and not children[node] and node not in new_leaves:
                        new_leaves.append(node)
            leaves = [n for n in new_leaves if not children[n]]
            first_round = False
    return parent, token, depth

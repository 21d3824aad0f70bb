"""Oracle of the host drafter: TEST INFRASTRUCTURE ONLY (imported by tests/ and by nothing else).

A plain, slow, obviously correct model of Cacheback's cache table and draft-tree growth, written
from the paper with Python lists, linear scans and sorting only -- no hash maps, no ordered dictionaries,
no code shared with the product's drafters (paper_2511_21699_amd/drafter.py, csrc/cb_drafter.cpp).

Section 3.1 (the cache table): pairs of a leader (LL tokens) and its followers (FL tokens each);
at most LC leaders and FC followers per leader; both domains evict their least recently used
entry, and "used" means inserted: an insertion makes its leader, and its follower under that
leader, the most recent one.
Section 3.2 (tree growth): starting from the last token of the context, the last LL tokens of a
root-to-leaf path are looked up, each follower found is attached under the leaf, and this repeats
breadth-first on the new leaves until no leaf has a follower or the tree holds TDL tokens; CRT
tokens of the budget are reserved for the rounds after the first.  Section 3.3: a frozen table is
used after the dynamic one and never changes.

The readings where the paper is silent are those the C header lists (most recent follower first,
token-by-token truncation at the budget and the depth cap, shared prefixes merged, a lookup during
growth counts as a use of the leader).  Pinned by tests/test_drafter_oracle.py.
"""
from __future__ import annotations


class TableOracle:
    def __init__(self, ll, fl, lc, fc):
        self.ll, self.fl, self.lc, self.fc = ll, fl, lc, fc
        self.frozen = False
        self.rows = []          # [leader tuple, [follower tuples]] ; both lists least recent first

    def _find(self, leader):
        for i, row in enumerate(self.rows):
            if row[0] == leader:
                return i
        return -1

    def insert(self, leader, follower):
        if self.frozen:
            return
        leader, follower = tuple(int(x) for x in leader), tuple(int(x) for x in follower)
        assert len(leader) == self.ll and len(follower) == self.fl
        i = self._find(leader)
        if i < 0:
            if len(self.rows) == self.lc:
                del self.rows[0]                       # the least recently used leader goes, followers and all
            self.rows.append([leader, [follower]])
            return
        row = self.rows.pop(i)
        self.rows.append(row)                          # now the most recent leader
        fols = row[1]
        if follower in fols:
            fols.remove(follower)
        elif len(fols) == self.fc:
            del fols[0]                                # this leader's least recently used follower goes
        fols.append(follower)

    def update(self, tokens, start=0):
        tokens = [int(x) for x in tokens]
        for i in range(len(tokens)):
            if i < self.ll or i < start or i + self.fl > len(tokens):
                continue
            self.insert(tokens[i - self.ll:i], tokens[i:i + self.fl])

    def query(self, leader, refresh=True):
        i = self._find(tuple(int(x) for x in leader))
        if i < 0:
            return []
        if refresh and not self.frozen:
            self.rows.append(self.rows.pop(i))
            i = len(self.rows) - 1
        return list(reversed(self.rows[i][1]))

    def size(self):
        return len(self.rows), sum(len(r[1]) for r in self.rows)


def grow_tree_oracle(context, tables, node_budget, depth_cap, crt=0):
    """Returns (parent, token, depth) lists; node 0 is the last token of the context."""
    context = [int(x) for x in context]
    parent, token, depth = [-1], [context[-1]], [0]

    def kids(n):
        return [i for i in range(len(parent)) if parent[i] == n]

    def last_tokens(n, count):
        seq = []
        while n != -1:
            seq.insert(0, token[n])
            n = parent[n]
        seq = context[:-1] + seq                      # the root path continues back into the context
        return seq[-count:] if len(seq) >= count else None

    for tab in tables:
        frontier = [i for i in range(len(parent)) if not kids(i)]
        round_no = 0
        while frontier and len(parent) < node_budget:
            round_no += 1
            cap = node_budget - crt if (round_no == 1 and crt > 0) else node_budget
            if cap <= len(parent):
                cap = min(node_budget, len(parent) + 1)  # a round may always add one node
            reached = []
            for leaf in frontier:
                if len(parent) >= cap:
                    break
                key = last_tokens(leaf, tab.ll)
                if key is None:
                    continue
                for fol in tab.query(key):
                    at = leaf
                    for tk in fol:
                        if depth[at] >= depth_cap:
                            break
                        same = [k for k in kids(at) if token[k] == tk]
                        if same:
                            at = same[0]
                            continue
                        if len(parent) >= cap:
                            break
                        parent.append(at)
                        token.append(tk)
                        depth.append(depth[at] + 1)
                        at = len(parent) - 1
                    if at != leaf and not kids(at) and at not in reached:
                        reached.append(at)
            frontier = [n for n in reached if not kids(n)]
    return parent, token, depth


def build_frozen_oracle(tokens, ll, fl, lc, fc):
    """Section 4: the frozen table from a corpus sample -- the LC most frequent leaders (LL-grams) and,
    per leader, its FC most frequent followers (FL-grams that come right after it).  Counted over the
    windows (leader, follower) that fit in the sample; equal counts: the earlier first window wins.
    Counting is done by sorting the windows and measuring runs."""
    tokens = [int(x) for x in tokens]
    wins = []                                          # (leader, follower, position)
    for i in range(ll, len(tokens) - fl + 1):
        wins.append((tuple(tokens[i - ll:i]), tuple(tokens[i:i + fl]), i))

    def runs(items):                                   # items: (key, position) -> [(count, first position, key)]
        items = sorted(items)
        out = []
        for key, pos in items:
            if out and out[-1][2] == key:
                out[-1][0] += 1
            else:
                out.append([1, pos, key])
        return out

    leaders = runs([(w[0], w[2]) for w in wins])
    leaders.sort(key=lambda r: (-r[0], r[1]))
    t = TableOracle(ll, fl, lc, fc)
    for _, _, leader in reversed(leaders[:lc]):
        fols = runs([(w[1], w[2]) for w in wins if w[0] == leader])
        fols.sort(key=lambda r: (-r[0], r[1]))
        for _, _, fol in reversed(fols[:fc]):
            t.insert(leader, fol)
    t.frozen = True
    return t

// Host-side drafter of Cacheback decoding: the leader -> follower cache table with LRU eviction in
// both domains (Section 3.1 of the paper) and the breadth-first growth of the draft-token tree
// (Section 3.2), behind the C ABI of cacheback_drafter.h.  Serial host code, no GPU involved.
//
// Table layout: leaders live in `lc` fixed slots; a hash index maps a leader's tokens to its slot;
// the slots form a doubly linked list in recency order (index links, head = least recent).  Each
// slot owns `fc` follower cells and a small array naming the cells oldest first, so that both LRU
// domains are updated with a few moves and nothing is allocated per insertion except the hash
// index's own node.
#include <stdint.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <unordered_map>
#include <utility>
#include <vector>

#include "cacheback.h"
#include "cacheback_drafter.h"

namespace {

struct KeyRef {
  const int32_t* p;
  int32_t n;
};
struct KeyHash {
  size_t operator()(const KeyRef& k) const {
    uint64_t h = 1469598103934665603ull;  // FNV-1a over the tokens
    for (int i = 0; i < k.n; i++) {
      h ^= (uint32_t)k.p[i];
      h *= 1099511628211ull;
    }
    return (size_t)(h ^ (h >> 29));
  }
};
struct KeyEq {
  bool operator()(const KeyRef& a, const KeyRef& b) const {
    return a.n == b.n && memcmp(a.p, b.p, (size_t)a.n * 4) == 0;
  }
};

}  // namespace

struct cbd_table {
  int32_t ll, fl, lc, fc;
  bool frozen = false;
  std::vector<int32_t> key;    // [lc][ll] leader tokens
  std::vector<int32_t> prev, next;  // recency list over used slots
  int32_t head = -1, tail = -1;     // least / most recent leader
  std::vector<int32_t> nfol;   // followers held per slot
  std::vector<uint8_t> order;  // [lc][fc] follower cells, oldest first
  std::vector<int32_t> ftok;   // [lc][fc][fl] follower tokens
  int32_t used = 0;            // slots 0 .. used-1 have been handed out (none is ever returned: a full table evicts)
  int64_t followers = 0;
  std::unordered_map<KeyRef, int32_t, KeyHash, KeyEq> index;  // keys point into `key`

  void unlink(int32_t s) {
    if (prev[s] >= 0) next[prev[s]] = next[s]; else head = next[s];
    if (next[s] >= 0) prev[next[s]] = prev[s]; else tail = prev[s];
  }
  void push_recent(int32_t s) {
    prev[s] = tail;
    next[s] = -1;
    if (tail >= 0) next[tail] = s; else head = s;
    tail = s;
  }
  void touch(int32_t s) {
    if (tail == s) return;
    unlink(s);
    push_recent(s);
  }
  int32_t find(const int32_t* leader) const {
    auto it = index.find(KeyRef{leader, ll});
    return it == index.end() ? -1 : it->second;
  }
};

namespace {

// The tree under construction.  Children are kept as short (token, node) lists per node.
struct Tree {
  int32_t* parent;
  int32_t* token;
  int32_t* depth;
  int32_t n = 0;
  std::vector<std::vector<std::pair<int32_t, int32_t>>> children;
  int32_t child(int32_t node, int32_t tk) const {
    for (const auto& c : children[node])
      if (c.first == tk) return c.second;
    return -1;
  }
  int32_t add(int32_t par, int32_t tk) {
    const int32_t id = n++;
    parent[id] = par;
    token[id] = tk;
    depth[id] = par < 0 ? 0 : depth[par] + 1;
    children.emplace_back();
    if (par >= 0) children[par].emplace_back(tk, id);
    return id;
  }
};

// Last `need` tokens of the root path of `node`, continued back into the context before the root
// token; returns how many there are (fewer than `need` when the context is too short).
int32_t path_tokens(const Tree& t, int32_t node, int32_t need, const int32_t* context, int64_t n_ctx, int32_t* out) {
  int32_t got = 0;
  int32_t tmp[16];
  for (int32_t x = node; x >= 0 && got < need; x = t.parent[x]) tmp[got++] = t.token[x];
  const int64_t before_root = n_ctx - 1;
  const int32_t extra = (int32_t)std::min<int64_t>(need - got, before_root);
  int32_t k = 0;
  for (int32_t i = 0; i < extra; i++) out[k++] = context[before_root - extra + i];
  for (int32_t i = got - 1; i >= 0; i--) out[k++] = tmp[i];
  return k;
}

}  // namespace

extern "C" {

int cbd_table_create(int32_t ll, int32_t fl, int32_t lc, int32_t fc, cbd_table** out) {
  if (!out || ll < 1 || fl < 1 || lc < 1 || fc < 1 || ll > 16 || fl > 16 || fc > 64) return CB_EINVAL;
  cbd_table* t = new (std::nothrow) cbd_table();
  if (!t) return CB_EINVAL;
  t->ll = ll; t->fl = fl; t->lc = lc; t->fc = fc;
  t->key.assign((size_t)lc * ll, 0);
  t->prev.assign(lc, -1);
  t->next.assign(lc, -1);
  t->nfol.assign(lc, 0);
  t->order.assign((size_t)lc * fc, 0);
  t->ftok.assign((size_t)lc * fc * fl, 0);
  t->index.reserve((size_t)lc * 2);
  *out = t;
  return CB_OK;
}

void cbd_table_destroy(cbd_table* t) { delete t; }

int cbd_table_insert(cbd_table* t, const int32_t* leader, const int32_t* follower) {
  if (!t || !leader || !follower) return CB_EINVAL;
  if (t->frozen) return CB_OK;
  const int32_t ll = t->ll, fl = t->fl, fc = t->fc;
  int32_t s = t->find(leader);
  if (s < 0) {
    if (t->used < t->lc) {
      s = t->used++;
    } else {  // evict the least recently used leader with all its followers
      s = t->head;
      t->index.erase(KeyRef{&t->key[(size_t)s * ll], ll});
      t->unlink(s);
      t->followers -= t->nfol[s];
    }
    memcpy(&t->key[(size_t)s * ll], leader, (size_t)ll * 4);
    t->index.emplace(KeyRef{&t->key[(size_t)s * ll], ll}, s);
    t->push_recent(s);
    t->nfol[s] = 1;
    t->order[(size_t)s * fc] = 0;
    memcpy(&t->ftok[(size_t)s * fc * fl], follower, (size_t)fl * 4);
    t->followers += 1;
    return CB_OK;
  }
  t->touch(s);  // inserting refreshes the leader
  uint8_t* ord = &t->order[(size_t)s * fc];
  int32_t* cells = &t->ftok[(size_t)s * fc * fl];
  const int32_t n = t->nfol[s];
  for (int32_t i = 0; i < n; i++) {
    if (memcmp(&cells[(size_t)ord[i] * fl], follower, (size_t)fl * 4) == 0) {  // present: becomes the most recent
      const uint8_t c = ord[i];
      memmove(ord + i, ord + i + 1, (size_t)(n - 1 - i));
      ord[n - 1] = c;
      return CB_OK;
    }
  }
  uint8_t cell;
  if (n < fc) {
    cell = (uint8_t)n;  // cells fill up in order; they are only recycled once all are in use
    t->nfol[s] = n + 1;
    t->followers += 1;
    ord[n] = cell;
  } else {  // evict this leader's least recent follower
    cell = ord[0];
    memmove(ord, ord + 1, (size_t)(n - 1));
    ord[n - 1] = cell;
  }
  memcpy(&cells[(size_t)cell * fl], follower, (size_t)fl * 4);
  return CB_OK;
}

int cbd_table_update(cbd_table* t, const int32_t* tokens, int64_t n, int64_t start) {
  if (!t || (!tokens && n > 0) || n < 0) return CB_EINVAL;
  for (int64_t i = std::max<int64_t>(t->ll, start); i + t->fl <= n; i++) {
    const int rc = cbd_table_insert(t, tokens + i - t->ll, tokens + i);
    if (rc) return rc;
  }
  return CB_OK;
}

int cbd_table_query(cbd_table* t, const int32_t* leader, int32_t refresh, int32_t* followers, int32_t* count) {
  if (!t || !leader || !followers || !count) return CB_EINVAL;
  *count = 0;
  const int32_t s = t->find(leader);
  if (s < 0) return CB_OK;
  if (refresh && !t->frozen) t->touch(s);
  const int32_t n = t->nfol[s], fl = t->fl;
  const uint8_t* ord = &t->order[(size_t)s * t->fc];
  const int32_t* cells = &t->ftok[(size_t)s * t->fc * fl];
  for (int32_t i = 0; i < n; i++) memcpy(followers + (size_t)i * fl, &cells[(size_t)ord[n - 1 - i] * fl], (size_t)fl * 4);
  *count = n;
  return CB_OK;
}

int cbd_table_build_frozen(int32_t ll, int32_t fl, int32_t lc, int32_t fc, const int32_t* tokens, int64_t n,
                           cbd_table** out) {
  if (!out || (!tokens && n > 0) || n < 0) return CB_EINVAL;
  cbd_table* t = nullptr;
  const int rc = cbd_table_create(ll, fl, lc, fc, &t);
  if (rc) return rc;
  struct Stat {
    int64_t count = 0, first = 0;
    std::unordered_map<KeyRef, std::pair<int64_t, int64_t>, KeyHash, KeyEq> followers;  // -> (count, first window)
  };
  std::unordered_map<KeyRef, Stat, KeyHash, KeyEq> leaders;  // keys point into `tokens`
  for (int64_t i = ll; i + fl <= n; i++) {
    Stat& st = leaders[KeyRef{tokens + i - ll, ll}];
    if (st.count++ == 0) st.first = i;
    auto& f = st.followers[KeyRef{tokens + i, fl}];
    if (f.first++ == 0) f.second = i;
  }
  // more frequent first, then earlier first window
  std::vector<std::pair<KeyRef, const Stat*>> top;
  top.reserve(leaders.size());
  for (const auto& kv : leaders) top.emplace_back(kv.first, &kv.second);
  std::sort(top.begin(), top.end(), [](const auto& a, const auto& b) {
    return a.second->count != b.second->count ? a.second->count > b.second->count : a.second->first < b.second->first;
  });
  if ((int64_t)top.size() > lc) top.resize((size_t)lc);
  std::vector<std::pair<KeyRef, std::pair<int64_t, int64_t>>> fols;
  for (size_t r = top.size(); r-- > 0;) {  // least frequent leader first (recency is irrelevant once frozen)
    fols.assign(top[r].second->followers.begin(), top[r].second->followers.end());
    std::sort(fols.begin(), fols.end(), [](const auto& a, const auto& b) {
      return a.second.first != b.second.first ? a.second.first > b.second.first : a.second.second < b.second.second;
    });
    if ((int64_t)fols.size() > fc) fols.resize((size_t)fc);
    for (size_t k = fols.size(); k-- > 0;)  // least frequent follower first: the most frequent ends up most recent
      cbd_table_insert(t, top[r].first.p, fols[k].first.p);
  }
  t->frozen = true;
  *out = t;
  return CB_OK;
}

int cbd_table_freeze(cbd_table* t) {
  if (!t) return CB_EINVAL;
  t->frozen = true;
  return CB_OK;
}

int cbd_table_size(const cbd_table* t, int64_t* leaders, int64_t* followers) {
  if (!t || !leaders || !followers) return CB_EINVAL;
  *leaders = (int64_t)t->index.size();
  *followers = t->followers;
  return CB_OK;
}

int cbd_grow_tree(cbd_table* const* tables, int32_t num_tables, const int32_t* context, int64_t n_ctx,
                  int32_t node_budget, int32_t depth_cap, int32_t crt, int32_t* parent, int32_t* token,
                  int32_t* depth, int32_t* n_nodes) {
  if (!tables || num_tables < 0 || !context || n_ctx < 1 || node_budget < 1 || depth_cap < 0 || crt < 0 || !parent ||
      !token || !depth || !n_nodes)
    return CB_EINVAL;
  for (int32_t i = 0; i < num_tables; i++)
    if (!tables[i]) return CB_EINVAL;
  Tree tr;
  tr.parent = parent;
  tr.token = token;
  tr.depth = depth;
  tr.children.reserve((size_t)node_budget);
  tr.add(-1, context[n_ctx - 1]);
  std::vector<int32_t> leaves, grown;
  std::vector<int32_t> seen((size_t)node_budget, -1);  // round in which a node was listed as a new leaf
  std::vector<int32_t> fols;
  int32_t key[16];
  int32_t round_id = 0;
  for (int32_t ti = 0; ti < num_tables; ti++) {
    cbd_table* tb = tables[ti];
    const int32_t ll = tb->ll, fl = tb->fl;
    fols.resize((size_t)tb->fc * fl);
    leaves.clear();
    for (int32_t i = 0; i < tr.n; i++)
      if (tr.children[i].empty()) leaves.push_back(i);
    bool first_round = true;
    while (!leaves.empty() && tr.n < node_budget) {
      // the chaining-reserved tokens keep part of the budget for the second and deeper rounds
      int32_t limit = (first_round && crt > 0) ? node_budget - crt : node_budget;
      limit = std::max(limit, std::min(node_budget, tr.n + 1));
      grown.clear();
      round_id++;
      for (int32_t leaf : leaves) {
        if (tr.n >= limit) break;
        if (path_tokens(tr, leaf, ll, context, n_ctx, key) < ll) continue;
        int32_t cnt = 0;
        cbd_table_query(tb, key, 1, fols.data(), &cnt);
        for (int32_t f = 0; f < cnt; f++) {
          int32_t node = leaf;
          for (int32_t j = 0; j < fl; j++) {
            if (tr.depth[node] >= depth_cap) break;
            const int32_t tk = fols[(size_t)f * fl + j];
            int32_t nxt = tr.child(node, tk);
            if (nxt < 0) {  // followers that share a prefix share the nodes
              if (tr.n >= limit) break;
              nxt = tr.add(node, tk);
            }
            node = nxt;
          }
          if (node != leaf && tr.children[node].empty() && seen[node] != round_id) {
            seen[node] = round_id;
            grown.push_back(node);
          }
        }
      }
      leaves.clear();
      for (int32_t x : grown)
        if (tr.children[x].empty()) leaves.push_back(x);
      first_round = false;
    }
  }
  *n_nodes = tr.n;
  return CB_OK;
}

}  // extern "C"

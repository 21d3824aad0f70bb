/*
 * cacheback_drafter.h -- C ABI of the host-side drafter of Cacheback decoding (arXiv 2511.21699).
 *
 * The drafter is serial host code (the paper, Section 1: drafting takes microseconds): a cache
 * table of leader -> follower n-grams with LRU eviction in both domains (Section 3.1), and the
 * breadth-first growth of the draft-token tree by recursive table queries (Section 3.2).  Its
 * trees are the input of cb_verify_tree (cacheback.h).  Nothing here touches a GPU; every pointer
 * is host memory; after cbd_table_create only the table's hash index allocates (and
 * cbd_table_build_frozen, which counts n-grams in temporary maps).
 *
 * Readings where the paper is silent (they shape the trees, never the verified results):
 * a query returns followers most-recently-inserted first; re-inserting a follower that is present
 * refreshes its recency; followers are cut token by token at the node budget and the depth cap;
 * followers that share a prefix under the same leaf are merged trie-style; the chaining-reserved
 * tokens (CRT) hold back part of the budget in the first breadth-first round of a table.
 *
 * All functions return CB_OK (0) or CB_EINVAL (bad argument) / CB_ECAP (output would not fit), the
 * codes of cacheback.h.  A table is not thread-safe.
 */
#ifndef CACHEBACK_DRAFTER_H
#define CACHEBACK_DRAFTER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cbd_table cbd_table;

/* Section 3.1: a table of at most `lc` leaders of `ll` tokens, each with at most `fc` followers of
 * `fl` tokens.  All four >= 1; ll, fl <= 16; fc <= 64. */
int cbd_table_create(int32_t ll, int32_t fl, int32_t lc, int32_t fc, cbd_table **out);
void cbd_table_destroy(cbd_table *t);

/* Section 3.1, insertion: a new leader evicts the least recently used leader (with its followers)
 * when the table is full; inserting under an existing leader makes it the most recent leader; a
 * follower that is present becomes that leader's most recent follower, a new one evicts the
 * leader's least recent follower when the leader is full.  leader[ll], follower[fl].  A frozen
 * table ignores the call (Section 3.3). */
int cbd_table_insert(cbd_table *t, const int32_t *leader, const int32_t *follower);

/* Sliding-window update (Section 3.2, last paragraph; prompt initialisation, Section 3.3): inserts
 * (tokens[i-ll .. i), tokens[i .. i+fl)) for every i in [max(ll, start), n - fl], in increasing i. */
int cbd_table_update(cbd_table *t, const int32_t *tokens, int64_t n, int64_t start);

/* Followers of leader[ll], most recent first: *count of them, fl tokens each, written to
 * followers[fc*fl].  refresh != 0 makes the leader the most recent one (what a query during tree
 * growth does) unless the table is frozen. */
int cbd_table_query(cbd_table *t, const int32_t *leader, int32_t refresh, int32_t *followers, int32_t *count);

/* Section 3.3: a frozen table keeps answering queries but ignores insertions and recency. */
int cbd_table_freeze(cbd_table *t);

/* Section 4 (how the paper builds its frozen table from a corpus sample): over all windows
 * (tokens[i-ll .. i), tokens[i .. i+fl)), i in [ll, n - fl], the `lc` most frequent leaders are
 * kept, and for each of them its `fc` most frequent followers; among equally frequent n-grams the
 * one whose first window comes earlier in the sample wins.  The new table is frozen; a query returns
 * a leader's followers most frequent first. */
int cbd_table_build_frozen(int32_t ll, int32_t fl, int32_t lc, int32_t fc, const int32_t *tokens, int64_t n,
                           cbd_table **out);

/* Current numbers of leaders and of followers (over all leaders). */
int cbd_table_size(const cbd_table *t, int64_t *leaders, int64_t *followers);

/* Section 3.2: grows the draft-token tree under the last token of context[n_ctx] (node 0, the root,
 * is that token).  The tables are used in order (dynamic first, then frozen, Section 3.3); each
 * grows the tree breadth-first from the current leaves -- a leaf's key is the last ll tokens of its
 * root path, continued back into the context -- until no leaf has a follower or the tree holds
 * node_budget nodes (the paper's TDL, root included).  No node is deeper than depth_cap.  crt > 0
 * caps the first round of each table at node_budget - crt nodes.
 * Outputs parent[], token[], depth[] (room for node_budget entries each; parent[0] = -1,
 * parent[i] < i) and *n_nodes. */
int cbd_grow_tree(cbd_table *const *tables, int32_t num_tables, const int32_t *context, int64_t n_ctx,
                  int32_t node_budget, int32_t depth_cap, int32_t crt, int32_t *parent, int32_t *token,
                  int32_t *depth, int32_t *n_nodes);

#ifdef __cplusplus
}
#endif
#endif /* CACHEBACK_DRAFTER_H */

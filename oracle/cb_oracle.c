/*
 * CPU oracle for Cacheback tree verification -- TEST INFRASTRUCTURE, not a product path.
 *
 * Plain, slow, double-precision statements of what one verification step computes, written from
 * the paper (Cacheback, arXiv 2511.21699) and sharing no code with the HIP library:
 *
 *   cbo_attention_rows  Section 3.2, tree attention: a draft-tree node attends to the KV-cached
 *                       prefix and, among the tree nodes, only to its ancestors (and itself -- the
 *                       reading under which every root-to-leaf path is ordinary causal attention).
 *   cbo_argmax          the token the forward pass "generates" at each node: first maximum of the
 *                       node's logits row (greedy decoding).
 *   cbo_accept          Section 3.2, last paragraphs: the longest branch prefix whose draft tokens
 *                       equal what the model generates at their parents is accepted, and the pass
 *                       yields one more token after it (1 .. 1+longest-branch tokens per step).
 *   cbo_compact         keeping the accepted nodes' K/V: cache slot S+j receives slot S+path[j].
 *                       (The paper itself re-feeds accepted tokens, Section 3.2; compaction is the
 *                       equivalent cache-side statement: afterwards the cache holds exactly the
 *                       accepted sequence.)
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call this file.
 * Every function is pinned by tests that do not go through this code (brute force over
 * root-to-leaf paths, library attention on chain trees, numpy argmax, sequential greedy checks,
 * the worked example of the paper's Figure 2).
 *
 * Element types: dtype 0 = IEEE float32, 1 = bfloat16 bit patterns (uint16).  All arithmetic is
 * in double; inputs widen exactly.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double load_elem(const void *base, int dtype, int64_t idx) {
  if (dtype == 1) {
    uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
    float f;
    memcpy(&f, &bits, 4);
    return (double)f;
  }
  return (double)((const float *)base)[idx];
}

/* element index of (sequence, slot, kv head, 0) in the cache */
static int64_t slot_index(int seq, int64_t slot, int h, int Hkv, int D, int block_size,
                          int64_t capacity, const int32_t *block_table, int max_blocks) {
  if (block_size > 0) {
    int64_t blk = block_table[(int64_t)seq * max_blocks + slot / block_size];
    return ((blk * block_size + slot % block_size) * Hkv + h) * (int64_t)D;
  }
  return (((int64_t)seq * capacity + slot) * Hkv + h) * (int64_t)D;
}

int cbo_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/*
 * rows: nrows triples (sequence, query head, node-local index).  out: nrows x D doubles.
 * Visible keys of node i of sequence b: cache slots 0..S_b-1 and S_b + a for every a on the
 * parent chain from i up to the root, i included.
 */
int cbo_attention_rows(int dtype, int Hq, int Hkv, int D, int block_size, int64_t capacity,
                       const void *q, const void *k, const void *v, const int32_t *block_table,
                       int max_blocks, const int32_t *kv_len, const int32_t *node_offsets,
                       const int32_t *parent, double scale, int nrows, const int32_t *rows,
                       double *out, int nthreads) {
  int g = Hq / Hkv;
  int status = 0;
  if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
  for (int r = 0; r < nrows; r++) {
    int b = rows[3 * r], h = rows[3 * r + 1], i = rows[3 * r + 2];
    int S = kv_len[b], N = node_offsets[b + 1] - node_offsets[b];
    const int32_t *par = parent + node_offsets[b];
    int hk = h / g;
    int nvis_max = S + N;
    int64_t *vis = (int64_t *)malloc(sizeof(int64_t) * (size_t)nvis_max);
    double *w = (double *)malloc(sizeof(double) * (size_t)nvis_max);
    if (!vis || !w) { status = 1; free(vis); free(w); continue; }
    int nvis = 0;
    for (int j = 0; j < S; j++) vis[nvis++] = j;
    for (int a = i, steps = 0; a >= 0 && steps <= N; a = par[a], steps++) vis[nvis++] = (int64_t)S + a;
    int64_t qoff = (((int64_t)node_offsets[b] + i) * Hq + h) * (int64_t)D;
    double m = -INFINITY;
    for (int t = 0; t < nvis; t++) {
      int64_t ko = slot_index(b, vis[t], hk, Hkv, D, block_size, capacity, block_table, max_blocks);
      double s = 0.0;
      for (int d = 0; d < D; d++) s += load_elem(q, dtype, qoff + d) * load_elem(k, dtype, ko + d);
      s *= scale;
      w[t] = s;
      if (s > m) m = s;
    }
    double denom = 0.0;
    for (int t = 0; t < nvis; t++) { w[t] = exp(w[t] - m); denom += w[t]; }
    double *o = out + (int64_t)r * D;
    for (int d = 0; d < D; d++) o[d] = 0.0;
    for (int t = 0; t < nvis; t++) {
      int64_t vo = slot_index(b, vis[t], hk, Hkv, D, block_size, capacity, block_table, max_blocks);
      for (int d = 0; d < D; d++) o[d] += w[t] * load_elem(v, dtype, vo + d);
    }
    for (int d = 0; d < D; d++) o[d] /= denom;
    free(vis);
    free(w);
  }
  return status;
}

/* first maximum of each row, single left-to-right scan with a strict comparison */
void cbo_argmax(int dtype, const void *logits, int N, int64_t V, int32_t *out) {
  for (int i = 0; i < N; i++) {
    int64_t base = (int64_t)i * V;
    double best = load_elem(logits, dtype, base);
    int32_t arg = 0;
    for (int64_t t = 1; t < V; t++) {
      double x = load_elem(logits, dtype, base + t);
      if (x > best) { best = x; arg = (int32_t)t; }
    }
    out[i] = arg;
  }
}

/*
 * Greedy acceptance over one tree.  a[i] is the token generated at node i.  A non-root node c is
 * accepted when every node x on the chain from c up to (not including) the root has
 * tok[x] == a[parent[x]].  The result is the accepted node of greatest depth (lowest index among
 * equals); path[0..L] runs from the root to it; tokens[j] = a[path[j]], the last one being the
 * extra token the pass always yields.  Returns L (number of accepted draft tokens).
 */
int cbo_accept(const int32_t *parent, const int32_t *tok, const int32_t *a, int N,
               int32_t *path, int32_t *tokens) {
  int best = 0, best_depth = 0;
  for (int c = 1; c < N; c++) {
    int ok = 1, depth = 0;
    for (int x = c; parent[x] >= 0; x = parent[x]) {
      if (tok[x] != a[parent[x]]) ok = 0;
      depth++;
    }
    if (ok && depth > best_depth) { best = c; best_depth = depth; }
  }
  int x = best;
  for (int j = best_depth; j >= 0; j--) { path[j] = x; x = parent[x]; }
  for (int j = 0; j <= best_depth; j++) tokens[j] = a[path[j]];
  return best_depth;
}

/*
 * In a cache owned by the caller: slot S+j <- slot S+path[j] for j = 1..L, K and V, every KV head.
 * Sources are snapshotted first so the statement holds whatever the order of the copies.
 */
int cbo_compact(int elem_bytes, int Hkv, int D, int block_size, int64_t capacity, void *k, void *v,
                const int32_t *block_table, int max_blocks, int seq, int S, int L,
                const int32_t *path) {
  size_t row = (size_t)D * (size_t)elem_bytes;
  size_t tok_bytes = row * (size_t)Hkv;
  unsigned char *snap = (unsigned char *)malloc(2 * tok_bytes * (size_t)(L > 0 ? L : 1));
  if (!snap) return 1;
  void *kv[2] = {k, v};
  for (int which = 0; which < 2; which++)
    for (int j = 1; j <= L; j++)
      for (int h = 0; h < Hkv; h++) {
        int64_t src = slot_index(seq, (int64_t)S + path[j], h, Hkv, D, block_size, capacity, block_table, max_blocks);
        memcpy(snap + ((size_t)which * L + (j - 1)) * tok_bytes + (size_t)h * row,
               (unsigned char *)kv[which] + (size_t)src * elem_bytes, row);
      }
  for (int which = 0; which < 2; which++)
    for (int j = 1; j <= L; j++)
      for (int h = 0; h < Hkv; h++) {
        int64_t dst = slot_index(seq, (int64_t)S + j, h, Hkv, D, block_size, capacity, block_table, max_blocks);
        memcpy((unsigned char *)kv[which] + (size_t)dst * elem_bytes,
               snap + ((size_t)which * L + (j - 1)) * tok_bytes + (size_t)h * row, row);
      }
  free(snap);
  return 0;
}

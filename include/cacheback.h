/*
 * cacheback.h -- C ABI of libcacheback_verify.so: tree verification for Cacheback speculative
 * decoding (arXiv 2511.21699) on one AMD MI355X (gfx950).
 *
 * One decoding step of the paper (Section 3.2) drafts a tree of tokens on the host and then
 * verifies all of its branches in one forward pass of the model.  This library is the GPU side of
 * that verification for one attention layer plus the final logits:
 *
 *   cb_verify_tree   tree attention -- every tree node attends to the KV-cached prefix and to its
 *                    own ancestors in the draft tree (the tree attention of Section 3.2; a node
 *                    also sees itself, which makes every root-to-leaf path ordinary causal
 *                    attention) -- followed by the greedy acceptance of
 *                    Section 3.2: the token the model generates at a node is the first maximum of
 *                    the node's logits row; the longest branch prefix whose draft tokens equal what
 *                    was generated at their parents is accepted, and the pass always yields one
 *                    more token after it.
 *   cb_compact_kv    keeps the K/V of the accepted nodes: cache slot S+j receives slot S+path[j],
 *                    so that the cache afterwards holds exactly the accepted sequence.  (The
 *                    paper's prototype re-feeds accepted tokens instead, Section 3.2; this is the
 *                    cache-side equivalent that avoids recomputing them.)
 *
 * Conventions
 *   - Node 0 of every tree is the root: the last accepted token of the previous step, not yet
 *     attended to.  The model forward has already written the K/V of tree node i of sequence b into
 *     cache slot kv_len[b] + i.  Nodes are topologically ordered: tree_parent[0] = -1 and
 *     0 <= tree_parent[i] < i.  The node counts include the root (the paper's total draft length
 *     counts the non-cached token as well).
 *   - All tensors have their innermost dimension (head_dim or vocabulary) contiguous, 16-byte
 *     aligned base pointers, and live in DEVICE memory unless a parameter says "host".
 *   - The caller owns every tensor, the workspace and the stream.  The library owns only cb_ctx
 *     and a small pinned host buffer; it allocates no device memory.  cb_verify_tree never writes
 *     the cache; cb_compact_kv writes only slots S+1 .. S+L of each sequence.
 *   - Every function returns CB_OK or an error code, writes no outputs on error, and never aborts.
 *     Argument checks run on the host before any launch.  cb_last_error gives a text.
 *   - One context serves one stream at a time; calls on one context must not overlap.
 *   - Inputs are assumed finite (no NaN/Inf); results are unspecified otherwise.
 */
#ifndef CACHEBACK_H
#define CACHEBACK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cb_ctx cb_ctx; /* opaque */

enum { CB_F32 = 0, CB_BF16 = 1 }; /* element types: IEEE float32, bfloat16 */

enum {
  CB_OK = 0,
  CB_EINVAL = 1, /* null pointer, unsupported shape or type, bad batch                    */
  CB_ETREE = 2,  /* malformed tree: root parent != -1, parent not in [0,i), too deep        */
  CB_ECAP = 3,   /* more nodes than max_nodes, prefix + nodes beyond the cache, workspace   */
  CB_ESTATE = 4, /* cb_compact_kv without a preceding successful verify                     */
  CB_EHIP = 5    /* HIP runtime failure (no device, launch error); text via cb_last_error   */
};

enum { CB_LAYOUT_TOKEN_MAJOR = 0, /* [.., token, kv_head, head_dim] */
       CB_LAYOUT_HEAD_MAJOR = 1   /* [.., kv_head, token, head_dim] */ };

#define CB_MAX_NODES 256 /* nodes per tree (ancestor sets are 256-bit)         */
#define CB_MAX_BATCH 64  /* sequences per call                                  */
#define CB_MAX_LAYERS 64 /* cache layers per cb_compact_kv call                 */

typedef struct {            /* immutable after cb_init */
  int32_t num_q_heads;      /* Hq                                                         */
  int32_t num_kv_heads;     /* Hkv, divides Hq (grouped-query attention when smaller)     */
  int32_t head_dim;         /* D: 64 or 128                                               */
  int32_t qkv_dtype;        /* CB_F32 or CB_BF16: type of q, k, v and of the attention output */
  int32_t logits_dtype;     /* CB_F32 or CB_BF16                                          */
  int32_t max_batch;        /* <= CB_MAX_BATCH                                            */
  int32_t max_nodes;        /* per tree, root included, <= CB_MAX_NODES                   */
  int32_t max_depth;        /* deepest node allowed (edges from the root)                 */
  int32_t vocab_size;       /* V                                                          */
  int32_t block_size;       /* 0 = contiguous cache, else tokens per block of a paged cache */
  int32_t max_splits;       /* upper bound on KV-sequence splits per row; 0 = default (64) */
  float softmax_scale;      /* <= 0 means 1/sqrt(head_dim)                                */
} cb_config;

typedef struct {             /* one attention layer's cache (device memory owned by the caller) */
  void *k, *v;               /* contiguous, token-major: [B][capacity][Hkv][D]
                                contiguous, head-major : [B][Hkv][capacity][D]
                                paged, token-major     : [num_blocks][block_size][Hkv][D]
                                paged, head-major      : [num_blocks][Hkv][block_size][D]      */
  int64_t capacity_or_num_blocks;
  const int32_t *block_table; /* device [B][max_blocks_per_seq], logical block -> physical block;
                                 NULL for a contiguous cache.  Entries are not checked on the host;
                                 the kernels clamp them into the pool, so a bad table gives wrong
                                 numbers, never a fault.                                         */
  int32_t max_blocks_per_seq;
  int32_t layout;             /* CB_LAYOUT_*                                                    */
} cb_kv_layer;

/* Bytes of device workspace cb_init needs for this configuration.  Host only. */
int cb_workspace_bytes(const cb_config *cfg, size_t *bytes);

/* Creates a context on the current HIP device.  `workspace` is device memory of at least
 * cb_workspace_bytes() bytes, 256-byte aligned, which the context uses until cb_destroy.
 * Clears the workspace's counters on the default (null) stream and waits for that. */
int cb_init(const cb_config *cfg, void *workspace, size_t workspace_bytes, cb_ctx **out);

/* Host-only: how the attention stage (Section 3.2, tree attention over prefix + ancestors) would be
 * cut up for these lengths, without touching a device.  plan[0] = kernel family (1 scalar, 2 MFMA),
 * plan[1] = partial slots per output row (splits of the longest sequence), plan[2] = keys per split
 * (a multiple of 32; splits x keys covers the longest sequence, shorter sequences use fewer splits),
 * plan[3] = output rows per workgroup tile (1 for the scalar family), plan[4] = workgroups launched
 * that have keys to sweep.  forced_splits > 0 overrides the planner's split count (capped at the
 * configuration's max_splits), like the "splits" option.  All arrays are host memory.  CB_EINVAL on
 * a bad configuration or shape. */
int cb_plan_attention(const cb_config *cfg, int32_t batch, const int32_t *kv_len,
                      const int32_t *node_offsets, int32_t forced_splits, int32_t plan[5]);

/* Host-only argument check used by cb_verify_tree (exported so it can be exercised without a GPU):
 * shapes against the configuration, tree well-formedness, cache capacity.  `err`/`err_len` may be
 * NULL/0; otherwise a text is written on failure. */
int cb_check_verify_args(const cb_config *cfg, int32_t batch, const cb_kv_layer *kv,
                         const int32_t *kv_len, const int32_t *node_offsets,
                         const int32_t *tree_parent, char *err, size_t err_len);

/*
 * Verifies one draft tree per sequence (Section 3.2 of the paper).
 *   q               device [sumN][Hq][D]: queries of all tree nodes, sequences back to back
 *   kv              the layer's cache; slots [kv_len[b], kv_len[b]+N_b) hold the tree nodes' K/V
 *   kv_len          host [batch]: KV-cached prefix lengths S_b >= 0
 *   node_offsets    host [batch+1]: CSR offsets of each sequence's nodes, node_offsets[0] = 0
 *   tree_parent     host [sumN]: parent of each node as an index local to its tree, -1 at roots
 *   draft_tokens    host [sumN]: token id of each node (the root's entry is not used)
 *   logits          device [sumN][V]: the model's output row at each node
 *   attn_out        device [sumN][Hq][D], qkv_dtype: attention output of every node
 *   accepted_len    host [batch]: number of accepted draft tokens L_b, 0 .. max_depth
 *   accepted_tokens host [batch][max_depth+1]: L_b+1 tokens per sequence, the tokens generated
 *                   at the root and at each accepted node in order (the last is the extra token a
 *                   pass always yields); the remaining entries are set to -1
 * Siblings may carry the same token; among accepted nodes of equal depth the lowest index wins.
 * Returns when accepted_len and accepted_tokens have arrived in host memory.  That can be before the
 * launch on `hip_stream` (a hipStream_t, NULL = the null stream) has ended: the acceptance flags its
 * results to the waiting host while the attention is still merging its splits.  attn_out is
 * therefore complete in stream order, not on return: work enqueued on `hip_stream` afterwards sees
 * it, a host read needs a synchronisation of the stream first.  A later call of this library on
 * another stream waits for this one's launch by itself.  Option "full_sync" = 1 (cb_set_option)
 * makes every call synchronise the stream before it returns.
 */
int cb_verify_tree(cb_ctx *ctx, void *hip_stream, int32_t batch, const void *q,
                   const cb_kv_layer *kv, const int32_t *kv_len, const int32_t *node_offsets,
                   const int32_t *tree_parent, const int32_t *draft_tokens, const void *logits,
                   void *attn_out, int32_t *accepted_len, int32_t *accepted_tokens);

/*
 * Same computation with the tree and the results resident on the device and no synchronisation:
 * only launches are enqueued on `hip_stream` (suitable for stream capture into a HIP graph).
 * kv_len and node_offsets stay host arrays (they are shapes; they travel as kernel arguments).
 *   d_tree_parent, d_draft_tokens   device [sumN]
 *   d_accepted_len                  device [batch]
 *   d_accepted_tokens               device [batch][max_depth+1]
 * The tree's contents cannot be checked on the host here: a malformed parent entry is treated as
 * "child of the root", nodes deeper than max_depth are never accepted (their attention rows are
 * unspecified), and the status word returned by cb_device_status becomes non-zero; nothing faults.
 */
int cb_verify_tree_device(cb_ctx *ctx, void *hip_stream, int32_t batch, const void *q,
                          const cb_kv_layer *kv, const int32_t *kv_len,
                          const int32_t *node_offsets, const int32_t *d_tree_parent,
                          const int32_t *d_draft_tokens, const void *logits, void *attn_out,
                          int32_t *d_accepted_len, int32_t *d_accepted_tokens);

/*
 * Tree attention alone (Section 3.2: every node attends to the cached prefix, its ancestors and
 * itself), for the layers of a model below the last one: the arguments of cb_verify_tree_device
 * without tokens, logits and results.  Launches only; leaves the state of the last verify call
 * (what cb_compact_kv, cb_get_path and cb_get_argmax refer to) untouched.
 */
int cb_tree_attention_device(cb_ctx *ctx, void *hip_stream, int32_t batch, const void *q,
                             const cb_kv_layer *kv, const int32_t *kv_len,
                             const int32_t *node_offsets, const int32_t *d_tree_parent,
                             void *attn_out);

/*
 * cb_tree_attention_device for callers that cannot allocate: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  No context and no workspace: the configuration is
 * passed with every call, and the scratch memory the kernels need (split partials, merge tickets,
 * ancestor sets) is a fixed 32 MiB array inside the library's device image, which every GPU the
 * library runs on holds until the process ends.  The call allocates nothing on the host or the device
 * and only enqueues kernels on `hip_stream`.  A call whose shapes need more scratch than the array
 * holds returns CB_ECAP (text via cb_last_error(NULL)); of the five benchmark workloads the batched
 * ragged one is beyond it.  All calls on one GPU share the array, which keeps the last call's
 * contents (the counters that must start at zero are cleared by the call itself): calls that overlap
 * on one GPU -- from different streams or threads -- race and give undefined results.  Results are
 * those of cb_tree_attention_device for the same arguments.
 */
int cb_tree_attention_noalloc(const cb_config *cfg, void *hip_stream, int32_t batch, const void *q,
                              const cb_kv_layer *kv, const int32_t *kv_len,
                              const int32_t *node_offsets, const int32_t *d_tree_parent,
                              void *attn_out);

/*
 * Moves the K/V of the path accepted by the last verify call of this context into place, for
 * `num_layers` caches that share one geometry (capacity, block table, layout) and differ only in
 * their k/v pointers: for j = 1..L_b, slot S_b+j <- slot S_b+path_b[j].  Enqueues on `hip_stream`.
 *   new_kv_len   host [batch] or NULL: S_b + L_b + 1.  After cb_verify_tree it is filled without
 *                waiting; after cb_verify_tree_device filling it synchronises the stream.
 */
int cb_compact_kv(cb_ctx *ctx, void *hip_stream, int32_t num_layers, const cb_kv_layer *layers,
                  int32_t *new_kv_len);

/* Test hooks (each synchronises the stream of the last verify call).
 *   cb_get_path     host [batch][max_depth+1]: node indices of the accepted path, -1 padded
 *   cb_get_argmax   host [sumN]: first-maximum index of each logits row
 *   cb_device_status  0, or a bit mask: 1 = malformed parent entry seen, 2 = node deeper than max_depth,
 *                     16 = (informational) a split merge had to read partials across XCDs,
 *                     32 = (informational) a workgroup of a cooperative merge gave up waiting and left
 *                     its slice to the workgroup that completed the tile */
int cb_get_path(cb_ctx *ctx, int32_t *path);
int cb_get_argmax(cb_ctx *ctx, int32_t *argmax);
int cb_device_status(cb_ctx *ctx, int32_t *status);

/* ------------------------------------------------------------------------------------------------
 * Not part of the method: knobs and probes for tests and measurements.  None of them changes what
 * is computed.
 * ------------------------------------------------------------------------------------------------ */

/* Options; unknown names give CB_EINVAL.
 *   "splits"     force the number of KV-sequence splits (0 = automatic)
 *   "attn_impl"  0 = automatic, 1 = scalar kernel (at most 8 splits on a configuration the MFMA kernel
 *                takes), 2 = MFMA kernel (bf16, head_dim 128 only)
 *   "stages"     bit mask of the steps cb_verify_tree_device enqueues (1 ancestor sets, 2 attention,
 *                4 argmax, 8 acceptance; default 15) -- for timing one step in isolation; with a
 *                step left out the results of the call are those of an earlier call or undefined
 *   "parallel_scan"  1 = run the logits scan on the context's second stream beside the attention
 *   "fuse_logits"    0 = never run the logits scan and the acceptance inside the attention launch
 *                    (default 1: small calls -- MFMA attention, sequences of at most 64/g nodes, bf16
 *                    logits, no more logits chunks than attention workgroups -- are one launch)
 *   "coop_merge"     0 = never merge the splits cooperatively (default 1: a grid that fits the
 *                    machine in one round has every workgroup of a tile merge a slice of it; otherwise,
 *                    and with 0, the last workgroup of a tile to finish merges it, or a merge kernel)
 *   "merge_spin_limit"  how often a workgroup of a cooperative merge polls for the tile's other
 *                    splits before it leaves its slice to the workgroup that completes the tile
 *                    (default 256; 0 makes every workgroup but the completing one give up at once)
 *   "full_sync"      1 = cb_verify_tree synchronises its stream before returning (default 0: it
 *                    returns when the results have arrived, see there)
 *   "external_merge" 1 = always merge with the separate merge kernel
 *   "timeline"       1 = launch the timeline build of the MFMA kernels (see cb_debug_timestamps)
 *   "time_attention"  1 = record HIP events around the attention kernels (see cb_last_attention_ms) */
int cb_set_option(cb_ctx *ctx, const char *name, int64_t value);

/* Time in milliseconds the attention kernels of the last verify call took on the device (HIP
 * events recorded around them on the call's stream); enabled with option "time_attention" = 1.
 * Synchronises.  Not available under stream capture. */
int cb_last_attention_ms(cb_ctx *ctx, float *ms);

/* How the last verify call was launched (host memory, no device access): info[0] = attention kernel
 * family (1 scalar, 2 MFMA), info[1] = partial slots per output row, info[2] = keys per split,
 * info[3] = 1 if the logits scan and the acceptance ran inside the attention launch, else 0,
 * info[4] = how the splits were merged (0 one split, 1 cooperatively by the tile's workgroups, 2 by the
 * last workgroup of a tile to finish, 3 by a separate merge kernel), info[5] = kernels the call
 * enqueued.  CB_ESTATE before the first verify call. */
int cb_last_launch_info(cb_ctx *ctx, int32_t info[6]);

/* With option "timeline" = 1 the MFMA attention runs in a build that stamps 100 MHz clock readings
 * per workgroup (entry, arguments read, loads issued, first stage ready, key sweep done, partials
 * written, merge may start, merge done; eight more for the logits work or the merge's phases).
 * Copies those of the first `workgroups` (<= 1024) rows of the last launch to host memory, 8 values
 * each: rows 0..511 the attention's, rows 512.. the second set of workgroups 0..511. */
int cb_debug_timestamps(cb_ctx *ctx, uint64_t *out, int32_t workgroups);

/* Enqueues a plain streaming read of `bytes` (a multiple of 16, 16-byte aligned) of device memory at
 * d_src -- 1024 workgroups, 16-byte loads, nothing else -- so that a benchmark can time what this
 * machine delivers for a bare read of the size the attention sweeps.  d_sink: 256 dwords of device
 * memory (practically never written).  No context needed. */
int cb_probe_stream_read(void *hip_stream, const void *d_src, int64_t bytes, uint32_t *d_sink);

const char *cb_last_error(const cb_ctx *ctx); /* "" when the last call succeeded; ctx may be NULL
                                                 for the error of a failed cb_init */
void cb_destroy(cb_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* CACHEBACK_H */

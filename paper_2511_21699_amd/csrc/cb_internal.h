// Internal declarations shared by the host API and the kernel translation units (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "cacheback.h"

namespace cb {

constexpr int kAncWords = CB_MAX_NODES / 32;  // 256-bit ancestor set per node
constexpr int kArgmaxChunk = 8192;            // logits elements scanned by one workgroup
constexpr int kRowTile = 64;                  // query rows per workgroup in the MFMA attention
constexpr int kCoopTiles = 512;               // tiles a cooperative split merge can serve (it needs the grid resident at once)
constexpr int kCoopTicketStride = 4096;       // bytes between their ticket words
// floats per (row, split) partial softmax state: o[D] unnormalised, m, l, padded to 16 bytes
constexpr int partial_stride(int D) { return D + 4; }

// Per-sequence shapes; passed to kernels by value (kernel arguments), so they need no upload and
// are captured with the launch.
struct SeqMeta {
  int32_t kv_len[CB_MAX_BATCH];
  int32_t node_off[CB_MAX_BATCH + 1];
  int32_t by_length[CB_MAX_BATCH];  // the sequences ordered by kv_len + nodes, longest first (filled by the host)
};

// Shapes of sequence `b` (uniform in the wave) without a dependent scalar load: every lane fetches
// "its" entry of the argument arrays with one vector load issued at kernel start, and the wanted
// entry is picked with readlane once b is known.  A chain of scalar loads, each waiting for the
// one before, costs about a microsecond per link at the start of every workgroup.
struct SeqShape {
  int S, off, N;
};
struct SeqMetaLanes {
  int kv, o0, o1, ord;
};
__device__ __forceinline__ SeqMetaLanes seq_meta_prefetch(const SeqMeta& meta) {
  const int lane = threadIdx.x & 63;
  SeqMetaLanes r;
  r.kv = meta.kv_len[lane];
  r.o0 = meta.node_off[lane];
  r.o1 = meta.node_off[lane + 1];
  r.ord = meta.by_length[lane];
  return r;
}
__device__ __forceinline__ SeqShape seq_shape(const SeqMetaLanes& m, int b) {
  SeqShape s;
  s.S = __builtin_amdgcn_readlane(m.kv, b);
  s.off = __builtin_amdgcn_readlane(m.o0, b);
  s.N = __builtin_amdgcn_readlane(m.o1, b) - s.off;
  return s;
}

// How to find cache slot (sequence, slot, kv head) in one layer; strides in elements.
struct KvAddr {
  const void* k;
  const void* v;
  const int32_t* block_table;
  int64_t seq_stride;    // contiguous: per sequence; paged: per physical block
  int64_t token_stride;
  int64_t head_stride;
  int64_t num_blocks;    // paged: pool size (block ids are clamped into it)
  int32_t max_blocks;    // paged: row length of the block table
  int32_t block_size;    // 0 = contiguous
};

__device__ __forceinline__ int64_t slot_offset(const KvAddr& a, int seq, int slot, int head) {
  if (a.block_size > 0) {
    int lb = slot / a.block_size;
    int64_t blk = a.block_table[(int64_t)seq * a.max_blocks + lb];
    blk = blk < 0 ? 0 : (blk >= a.num_blocks ? a.num_blocks - 1 : blk);
    return blk * a.seq_stride + (int64_t)(slot - lb * a.block_size) * a.token_stride +
           (int64_t)head * a.head_stride;
  }
  return (int64_t)seq * a.seq_stride + (int64_t)slot * a.token_stride + (int64_t)head * a.head_stride;
}

// Ancestor sets of one tree built inside a workgroup (any block size >= 256; the first 256 threads
// own one node each).  Section 3.2 of the paper: a tree token attends only to its ancestors (and, in
// this library's reading, itself); anc[i] is the 256-bit set {i, parent(i), parent(parent(i)), ...}.
// Pointer jumping: after r rounds a node knows its 2^r nearest ancestors (itself included), so
// jump_rounds(max_depth) rounds complete every node of depth <= max_depth, and eight rounds any
// tree of up to 256 nodes.  `parent_of` is the node's sanitised parent (-1 at the root) for
// threads < N.  On return anc[i][0..7] holds node i's set for every i < N, all threads have passed
// a barrier, and the return value is the thread's remaining jump pointer: >= 0 exactly when its
// node has more ancestors than the rounds could collect (its set is then incomplete).  The barriers are bare s_barrier instructions (LDS traffic is
// ordered by explicit lgkmcnt waits), so the routine can run while global->LDS loads are in flight.
struct AncScratch {
  uint32_t anc[CB_MAX_NODES][kAncWords];
  int jump[CB_MAX_NODES];
};
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}
__host__ __device__ __forceinline__ int jump_rounds(int max_depth) {
  int r = 0;
  while (r < 8 && (1 << r) < max_depth + 1) r++;
  return r;
}
__device__ __forceinline__ int build_ancestor_sets(AncScratch& sh, int N, int parent_of, int rounds) {
  const int t = threadIdx.x;
  uint32_t mine[kAncWords];
  int j = -1;
  if (t < CB_MAX_NODES) {
#pragma unroll
    for (int w = 0; w < kAncWords; w++) mine[w] = (t < N && (t >> 5) == w) ? (1u << (t & 31)) : 0u;
    j = t < N ? parent_of : -1;
#pragma unroll
    for (int w = 0; w < kAncWords; w++) sh.anc[t][w] = mine[w];
    sh.jump[t] = j;
  }
  for (int r = 0; r < rounds; r++) {
    lds_barrier();
    uint32_t other[kAncWords];
    int jj = -1;
    if (t < CB_MAX_NODES && j >= 0) {
#pragma unroll
      for (int w = 0; w < kAncWords; w++) other[w] = sh.anc[j][w];
      jj = sh.jump[j];
    }
    lds_barrier();
    if (t < CB_MAX_NODES && j >= 0) {
#pragma unroll
      for (int w = 0; w < kAncWords; w++) {
        mine[w] |= other[w];
        sh.anc[t][w] = mine[w];
      }
      j = jj;
      sh.jump[t] = j;
    }
  }
  lds_barrier();
  return j;
}

// Parent of node t of a tree as the kernels use it: -1 at the root, entries outside [0, t) become
// 0 ("child of the root"), and the status word gets bit 0 when an entry had to be repaired.
__device__ __forceinline__ int sanitized_parent(const int32_t* parent, int off, int t, int32_t* status) {
  if (t == 0) {
    if (parent[off] != -1 && status) atomicOr(status, 1);
    return -1;
  }
  int p = parent[off + t];
  if (p < 0 || p >= t) {
    if (status) atomicOr(status, 1);
    p = 0;
  }
  return p;
}

struct AttnParams {
  const void* q;     // [sumN][Hq][D]
  void* out;         // [sumN][Hq][D]
  KvAddr kv;
  const uint32_t* anc;  // [sumN][kAncWords] (scalar kernel; the MFMA kernel builds the sets itself)
  const int32_t* parent;  // [sumN] device tree, local parent indices
  float* partial;       // split partials; scalar kernel: [sumN*Hq][nsplit][partial_stride(D)]: o[D] (unnormalised), m, l, pad;
                        // the MFMA kernel has its own bf16 layout (cb_attn_mfma.hip)
  uint32_t* tickets;    // two 64-bit words per (sequence, kv head, row tile): ticket, splits that gave up waiting
  uint32_t* coop_tickets;  // cooperative merge: kCoopTiles stretches of kCoopTicketStride bytes, two 64-bit words used in each
  int32_t Hq, Hkv, D;
  int32_t chunk;        // keys per split
  int32_t nsplit;       // partial slots per row (>= splits any sequence uses)
  int32_t batch;
  float scale;
  int32_t xcd_remap;    // 1: renumber workgroups so that all splits of a tile run on one XCD; 2: and every XCD takes
                        // its share -- a fixed set of (kv head, row tile) pairs of all sequences -- longest sequence first
  int32_t grid_x, grid_y, grid_z;  // launch grid, repeated here so the kernel reads one argument block
  int32_t external_merge;  // 1: the kernel only writes partials; launch_attn_mfma runs a merge kernel afterwards
  int32_t coop_merge;      // 1: every workgroup of a tile merges a slice of it after a bounded wait for the others
                           // (set by the launcher when the grid is resident in one round); -1 on input: never
  int32_t spin_limit;      // cooperative merge: polls of the tile's ticket before a workgroup gives up
  int32_t max_depth;    // deepest node the configuration allows (bounds the ancestor-set rounds)
  int32_t timeline;     // 1: launch the timeline build of the kernel (stamps per workgroup in dbg_ts; a measurement aid)
  int32_t force_external_merge;  // 1: always merge with the separate kernel (a test aid)
  int32_t* status;      // device status word (bit 4: a merge had to use cross-XCD loads)
  unsigned long long* dbg_ts;  // timeline build: 8 timestamps (100 MHz) per workgroup, 1024 rows
};

struct ArgmaxPartial {
  float value;
  int32_t index;
};

// ---- launchers (defined in the .hip files); all enqueue on `st` and return the launch status
hipError_t launch_tree_prepare(hipStream_t st, int batch, const SeqMeta& meta, const int32_t* parent,
                               int max_depth, uint32_t* anc, int32_t* status);
// zeroes `run` 64-bit words at each of `count` places `stride` words apart
hipError_t launch_zero_words(hipStream_t st, unsigned long long* base, int count, int stride, int run);
// scans the logits; with prep_parent != nullptr the same launch also builds the ancestor sets
hipError_t launch_argmax(hipStream_t st, const void* logits, int dtype, int rows, int64_t V,
                         ArgmaxPartial* partial, int nchunks, int batch, const SeqMeta& meta,
                         const int32_t* prep_parent, int max_depth, uint32_t* prep_anc, int32_t* status);
struct AcceptArgs;  // cb_logits.h
struct LogitsWork;
hipError_t launch_accept(hipStream_t st, int batch, const SeqMeta& meta, const AcceptArgs& args);
hipError_t launch_compact(hipStream_t st, int batch, const SeqMeta& meta, const KvAddr* layers,
                          int num_layers, int Hkv, int D, int elem_bytes, int max_depth,
                          const int32_t* path, const int32_t* acc_len, int32_t* new_len);
hipError_t launch_attn_simt(hipStream_t st, const AttnParams& p, const SeqMeta& meta, int dtype,
                            int max_nodes_in_call);
hipError_t launch_merge(hipStream_t st, const AttnParams& p, const SeqMeta& meta, int dtype, int total_nodes);
int attn_mfma_tile_rows(int mrows);            // rows per workgroup tile chosen for a given g*N
// bytes the MFMA path's partial states can take (its own layout, padded to 16-row tiles per kv head)
size_t attn_mfma_partial_bytes(size_t max_total_nodes, int Hq, int Hkv, int max_batch, int max_splits);
bool attn_mfma_supports(const AttnParams& p);  // shape/geometry the MFMA kernel takes (bf16 is the caller's check)
bool attn_mfma_can_fuse(const AttnParams& p, int max_nodes_in_call, int64_t logits_items, int logits_dtype);
// with logits_work != nullptr (only if attn_mfma_can_fuse) the same launch also scans the logits and runs the acceptance
// merge_kind (may be null): 0 one split, 1 cooperative merge, 2 merge by the last workgroup to arrive, 3 merge kernel
hipError_t launch_attn_mfma(hipStream_t st, const AttnParams& p, const SeqMeta& meta, int max_nodes_in_call,
                            int total_nodes, const LogitsWork* logits_work, int* merge_kind);

}  // namespace cb

// Tree preparation (ancestor sets), vocabulary argmax, greedy acceptance and KV compaction kernels.
// gfx950 only; 64-wide wavefronts are assumed throughout.
#include "cb_logits.h"

namespace cb {

// ------------------------------------------------------------------------------------------------
// Ancestor sets.  Section 3.2 of the paper: a tree token attends only to its ancestors (and, in
// this library's reading, itself).  anc[i] is the 256-bit set {i, parent(i), parent(parent(i)), ...}.
// Built by pointer jumping in LDS: after r rounds a node knows its 2^r nearest ancestors, so eight
// rounds cover any tree of up to 256 nodes whatever its depth.
// ------------------------------------------------------------------------------------------------
struct PrepareLds {
  uint32_t A[2][CB_MAX_NODES][kAncWords];
  int J[2][CB_MAX_NODES];
};

__device__ __forceinline__ void tree_prepare_block(PrepareLds& sh, const SeqMeta& meta, int b,
                                                   const int32_t* __restrict__ parent, int max_depth,
                                                   uint32_t* __restrict__ anc, int32_t* status) {
  auto& A = sh.A;
  auto& J = sh.J;
  const int t = threadIdx.x;
  const int off = meta.node_off[b];
  int N = meta.node_off[b + 1] - off;
  N = N > CB_MAX_NODES ? CB_MAX_NODES : N;
  int p = -1;
  if (t < N) p = sanitized_parent(parent, off, t, status);
#pragma unroll
  for (int w = 0; w < kAncWords; w++) A[0][t][w] = (t < N && (t >> 5) == w) ? (1u << (t & 31)) : 0u;
  J[0][t] = p;
  for (int r = 0; r < 8; r++) {
    __syncthreads();
    const int cur = r & 1, nxt = cur ^ 1;
    const int j = J[cur][t];
#pragma unroll
    for (int w = 0; w < kAncWords; w++) A[nxt][t][w] = A[cur][t][w] | (j >= 0 ? A[cur][j][w] : 0u);
    J[nxt][t] = j >= 0 ? J[cur][j] : -1;
  }
  __syncthreads();
  if (t < N) {
    int depth = -1;
#pragma unroll
    for (int w = 0; w < kAncWords; w++) {
      uint32_t x = A[0][t][w];  // 8 rounds: the result is back in buffer 0
      depth += __popc(x);
      anc[(int64_t)(off + t) * kAncWords + w] = x;
    }
    if (depth > max_depth && status) atomicOr(status, 2);
  }
}

__global__ __launch_bounds__(256) void k_tree_prepare(SeqMeta meta, const int32_t* __restrict__ parent,
                                                      int max_depth, uint32_t* __restrict__ anc,
                                                      int32_t* status) {
  __shared__ PrepareLds sh;
  tree_prepare_block(sh, meta, blockIdx.x, parent, max_depth, anc, status);
}

// Zero-fill of `count` 64-bit words, `stride` words apart, `run` words at each place (counters that
// must start at zero; a kernel rather than a memset so that the call can be captured into a graph).
__global__ __launch_bounds__(256) void k_zero_words(unsigned long long* base, int count, int stride, int run) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < count * run) base[(int64_t)(i / run) * stride + i % run] = 0ull;
}

hipError_t launch_zero_words(hipStream_t st, unsigned long long* base, int count, int stride, int run) {
  if (count <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_zero_words, dim3((count * run + 255) / 256), dim3(256), 0, st, base, count, stride, run);
  return hipGetLastError();
}

hipError_t launch_tree_prepare(hipStream_t st, int batch, const SeqMeta& meta, const int32_t* parent,
                               int max_depth, uint32_t* anc, int32_t* status) {
  hipLaunchKernelGGL(k_tree_prepare, dim3(batch), dim3(256), 0, st, meta, parent, max_depth, anc, status);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Argmax over the vocabulary: the token the model generates at a node is the first maximum of the
// node's logits row.  One workgroup scans kArgmaxChunk elements (scan_chunk() of cb_logits.h).
// ------------------------------------------------------------------------------------------------
// Rows [0, rows) of the grid's y dimension scan logits; when `prep` is set, rows [rows, rows + batch)
// build the ancestor sets of one sequence each (x = 0 only), which saves a launch of their own.
struct PrepareArgs {
  const int32_t* parent;
  uint32_t* anc;
  int32_t* status;
  int32_t max_depth;
  int32_t enabled;
};

template <typename T>
__global__ __launch_bounds__(256) void k_argmax(const T* __restrict__ logits, int64_t V, int rows,
                                                ArgmaxPartial* __restrict__ out, int nchunks, SeqMeta meta,
                                                PrepareArgs prep) {
  __shared__ PrepareLds prep_lds;
  if ((int)blockIdx.y >= rows) {
    if (blockIdx.x == 0 && prep.enabled)
      tree_prepare_block(prep_lds, meta, blockIdx.y - rows, prep.parent, prep.max_depth, prep.anc, prep.status);
    return;
  }
  __shared__ ScanLds scan_lds;
  const int row = blockIdx.y, c = blockIdx.x;
  float bv;
  int bi;
  scan_chunk<T, 256>(logits + (int64_t)row * V, V, c, threadIdx.x, scan_lds, bv, bi);
  if (threadIdx.x == 0) amax_store<false>(out + (int64_t)row * nchunks + c, bv, bi);
}

hipError_t launch_argmax(hipStream_t st, const void* logits, int dtype, int rows, int64_t V,
                         ArgmaxPartial* partial, int nchunks, int batch, const SeqMeta& meta,
                         const int32_t* prep_parent, int max_depth, uint32_t* prep_anc, int32_t* status) {
  PrepareArgs prep;
  prep.parent = prep_parent;
  prep.anc = prep_anc;
  prep.status = status;
  prep.max_depth = max_depth;
  prep.enabled = prep_parent != nullptr;
  dim3 grid(nchunks, rows + (prep.enabled ? batch : 0));
  if (dtype == CB_BF16)
    hipLaunchKernelGGL(k_argmax<uint16_t>, grid, dim3(256), 0, st, (const uint16_t*)logits, V, rows, partial, nchunks, meta, prep);
  else
    hipLaunchKernelGGL(k_argmax<float>, grid, dim3(256), 0, st, (const float*)logits, V, rows, partial, nchunks, meta, prep);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Greedy acceptance (Section 3.2, last paragraphs), one workgroup per sequence; the arithmetic is
// accept_sequence() of cb_logits.h.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_accept(SeqMeta meta, AcceptArgs args) {
  __shared__ AcceptLds sh;
  const int b = blockIdx.x;
  const int off = meta.node_off[b], N = meta.node_off[b + 1] - off;
  if (N <= 64) {
    if (threadIdx.x < 64) accept_wave<false>(args, b, off, N);
  } else {
    accept_sequence<false>(sh, args, b, off, N);
  }
}

hipError_t launch_accept(hipStream_t st, int batch, const SeqMeta& meta, const AcceptArgs& args) {
  hipLaunchKernelGGL(k_accept, dim3(batch), dim3(256), 0, st, meta, args);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// KV compaction: slot S+j <- slot S+path[j], j = 1..L, for K and V of every kv head and layer.
// path[j] >= j and the path is increasing, so slot S+j can be the source of an earlier step.  One
// thread owns one 16-byte column (layer, K|V, head, offset in the row) and walks j upwards, eight
// steps at a time: every read of a slot happens before the same thread overwrites it, and no other
// thread touches the column.
// ------------------------------------------------------------------------------------------------
// The layers share their geometry; only the base pointers differ, so the kernel takes one KvAddr
// and two pointer tables.
struct LayerPtrs {
  void* k[CB_MAX_LAYERS];
  void* v[CB_MAX_LAYERS];
};

__global__ __launch_bounds__(256) void k_compact(SeqMeta meta, KvAddr geo, LayerPtrs ptrs, int Hkv,
                                                 int row_vecs, int elem_shift, int max_depth,
                                                 const int32_t* __restrict__ path,
                                                 const int32_t* __restrict__ acc_len,
                                                 int32_t* __restrict__ new_len) {
  const int b = blockIdx.z;
  const int layer = blockIdx.y >> 1, which = blockIdx.y & 1;
  // the accepted length and the first path entries are requested together, before either is used
  constexpr int kBatch = 8;
  const int32_t* prow = path + b * (max_depth + 1);
  int L = acc_len[b];
  int src[kBatch];
#pragma unroll
  for (int u = 0; u < kBatch; u++) src[u] = prow[1 + u <= max_depth ? 1 + u : max_depth];
  const int S = meta.kv_len[b];
  const int N = meta.node_off[b + 1] - meta.node_off[b];
  L = L < 0 ? 0 : (L > max_depth ? max_depth : L);
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) new_len[b] = S + L + 1;
  const int col = blockIdx.x * 256 + threadIdx.x;
  if (col >= Hkv * row_vecs) return;
  const int h = col / row_vecs, vec = col - h * row_vecs;
  char* base = reinterpret_cast<char*>(which ? ptrs.v[layer] : ptrs.k[layer]);
  // Steps j0+1 .. j0+kBatch at a time: all of a batch's reads are issued before its first write.
  // That is the serial order's result: step j reads slot S+path[j] >= S+j, which no earlier step
  // (they write slots below S+j) has touched, so every read wants the slot's original contents.
  for (int j0 = 0; j0 < L; j0 += kBatch) {
    if (j0 > 0) {
#pragma unroll
      for (int u = 0; u < kBatch; u++) src[u] = prow[j0 + 1 + u <= max_depth ? j0 + 1 + u : max_depth];
    }
    uint4 x[kBatch];
    bool live[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; u++) {
      const int j = j0 + 1 + u;
      // (src == j: nothing to move; src < j or >= N cannot happen for a path the acceptance produced)
      live[u] = j <= L && src[u] > j && src[u] < N;
      if (live[u]) {
        const int64_t so = slot_offset(geo, b, S + src[u], h);
        x[u] = *reinterpret_cast<const uint4*>(base + (so << elem_shift) + (int64_t)vec * 16);
      }
    }
#pragma unroll
    for (int u = 0; u < kBatch; u++) {
      if (live[u]) {
        const int64_t doff = slot_offset(geo, b, S + j0 + 1 + u, h);
        *reinterpret_cast<uint4*>(base + (doff << elem_shift) + (int64_t)vec * 16) = x[u];
      }
    }
  }
}

hipError_t launch_compact(hipStream_t st, int batch, const SeqMeta& meta, const KvAddr* layers,
                          int num_layers, int Hkv, int D, int elem_bytes, int max_depth,
                          const int32_t* path, const int32_t* acc_len, int32_t* new_len) {
  LayerPtrs ptrs;
  for (int l = 0; l < num_layers; l++) {
    ptrs.k[l] = const_cast<void*>(layers[l].k);
    ptrs.v[l] = const_cast<void*>(layers[l].v);
  }
  const int row_vecs = D * elem_bytes / 16;
  const int elem_shift = elem_bytes == 4 ? 2 : 1;  // KvAddr strides are in elements, the copy works in bytes
  const int cols = Hkv * row_vecs;
  dim3 grid((cols + 255) / 256, num_layers * 2, batch);
  hipLaunchKernelGGL(k_compact, grid, dim3(256), 0, st, meta, layers[0], ptrs, Hkv, row_vecs, elem_shift,
                     max_depth, path, acc_len, new_len);
  return hipGetLastError();
}

}  // namespace cb

// Tree preparation (ancestor sets), vocabulary argmax, greedy acceptance and KV compaction kernels.
// gfx950 only; 64-wide wavefronts are assumed throughout.
#include "cb_internal.h"

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

hipError_t launch_tree_prepare(hipStream_t st, int batch, const SeqMeta& meta, const int32_t* parent,
                               int max_depth, uint32_t* anc, int32_t* status) {
  hipLaunchKernelGGL(k_tree_prepare, dim3(batch), dim3(256), 0, st, meta, parent, max_depth, anc, status);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Argmax over the vocabulary: the token the model generates at a node is the first maximum of the
// node's logits row.  One workgroup scans kArgmaxChunk elements with 16-byte loads; (value, index)
// pairs are combined under the total order "larger value, then smaller index" at every level, so
// equal maxima (common with bf16 logits) resolve to the lowest index exactly as a serial scan does.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ float elem_to_float(float x) { return x; }
__device__ __forceinline__ float elem_to_float(uint16_t x) { return __uint_as_float(((uint32_t)x) << 16); }

__device__ __forceinline__ void amax_take(float& bv, int& bi, float v, int i) {
  if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
}

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
  constexpr int VEC = 16 / sizeof(T);
  constexpr int kVecPerThread = kArgmaxChunk / VEC / 256;
  const int row = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
  const int64_t start = (int64_t)c * kArgmaxChunk;
  const int64_t end = (start + kArgmaxChunk < V) ? start + kArgmaxChunk : V;
  const T* base = logits + (int64_t)row * V;
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  const bool aligned = ((reinterpret_cast<uintptr_t>(base + start)) & 15) == 0;
  int64_t vec_end = start;
  if (aligned) {
    const int64_t nvec = (end - start) / VEC;
    vec_end = start + nvec * VEC;
    const uint4* vp = reinterpret_cast<const uint4*>(base + start);
    uint4 u[kVecPerThread];  // all of the thread's loads are in flight together
#pragma unroll
    for (int k = 0; k < kVecPerThread; k++) {
      const int64_t i = tid + k * 256;
      u[k] = i < nvec ? vp[i] : uint4{0, 0, 0, 0};
    }
#pragma unroll
    for (int k = 0; k < kVecPerThread; k++) {
      const int64_t i = tid + k * 256;
      if (i >= nvec) continue;
      const int e0 = (int)(start + i * VEC);
      if constexpr (sizeof(T) == 2) {
        const uint32_t w[4] = {u[k].x, u[k].y, u[k].z, u[k].w};
#pragma unroll
        for (int j = 0; j < 4; j++) {
          amax_take(bv, bi, __uint_as_float(w[j] << 16), e0 + 2 * j);
          amax_take(bv, bi, __uint_as_float(w[j] & 0xffff0000u), e0 + 2 * j + 1);
        }
      } else {
        amax_take(bv, bi, __uint_as_float(u[k].x), e0);
        amax_take(bv, bi, __uint_as_float(u[k].y), e0 + 1);
        amax_take(bv, bi, __uint_as_float(u[k].z), e0 + 2);
        amax_take(bv, bi, __uint_as_float(u[k].w), e0 + 3);
      }
    }
  }
  for (int64_t i = vec_end + tid; i < end; i += 256) amax_take(bv, bi, elem_to_float(base[i]), (int)i);
  // wavefront, then workgroup
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) {
    float ov = __shfl_xor(bv, s, 64);
    int oi = __shfl_xor(bi, s, 64);
    amax_take(bv, bi, ov, oi);
  }
  __shared__ float sv[4];
  __shared__ int si[4];
  if ((tid & 63) == 0) { sv[tid >> 6] = bv; si[tid >> 6] = bi; }
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < 4; w++) amax_take(bv, bi, sv[w], si[w]);
    ArgmaxPartial r;
    r.value = bv;
    r.index = bi;
    out[(int64_t)row * nchunks + c] = r;
  }
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
// Greedy acceptance (Section 3.2, last paragraphs).  A node is accepted when every non-root node on
// its chain carries the token generated at that node's parent; with match = {x : tok[x] ==
// a[parent(x)]} (root included) that is anc[c] being a subset of match.  The accepted node of
// greatest depth wins (lowest index among equals); its ancestor set *is* the path, each member
// sitting at position depth(member) = |anc(member)| - 1.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_accept(SeqMeta meta, const int32_t* __restrict__ parent,
                                                const int32_t* __restrict__ tokens,
                                                int32_t* status,
                                                const ArgmaxPartial* __restrict__ partial, int nchunks,
                                                int max_depth, int32_t* __restrict__ argmax_out,
                                                int32_t* __restrict__ path, int32_t* len_ctx,
                                                int32_t* len_user, int32_t* __restrict__ tok_user) {
  __shared__ int sh_a[CB_MAX_NODES];
  __shared__ AncScratch sh_anc;
  __shared__ uint32_t sh_match[kAncWords];
  __shared__ uint32_t sh_best[kAncWords];
  __shared__ uint32_t sh_key[4];
  const int b = blockIdx.x, t = threadIdx.x;
  const int off = meta.node_off[b];
  int N = meta.node_off[b + 1] - off;
  N = N > CB_MAX_NODES ? CB_MAX_NODES : N;
  int a = -1;
  if (t < N) {
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int c = 0; c < nchunks; c++) {
      ArgmaxPartial r = partial[(int64_t)(off + t) * nchunks + c];
      amax_take(bv, bi, r.value, r.index);
    }
    a = bi;
    argmax_out[off + t] = a;
  }
  sh_a[t] = a;
  __syncthreads();
  bool match = false;
  int par = -1;
  if (t < N) {
    par = sanitized_parent(parent, off, t, status);
    match = (t == 0) || (tokens[off + t] == sh_a[par]);
  }
  build_ancestor_sets(sh_anc, N, par);  // (the attention kernels build their own; nothing is passed between them)
  const unsigned long long bal = __ballot(match);
  if ((t & 63) == 0) {
    sh_match[(t >> 6) * 2] = (uint32_t)bal;
    sh_match[(t >> 6) * 2 + 1] = (uint32_t)(bal >> 32);
  }
  __syncthreads();
  uint32_t my[kAncWords];
  int depth = -1;
  bool acc = t < N;
#pragma unroll
  for (int w = 0; w < kAncWords; w++) {
    my[w] = (t < N) ? sh_anc.anc[t][w] : 0u;
    depth += __popc(my[w]);
    acc = acc && ((my[w] & ~sh_match[w]) == 0u);
  }
  if (depth > max_depth) {
    acc = false;
    if (t < N) atomicOr(status, 2);
  }
  uint32_t key = acc ? ((uint32_t)(depth + 1) << 16) | (uint32_t)(0xffff - t) : 0u;
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) {
    uint32_t o = __shfl_xor(key, s, 64);
    key = o > key ? o : key;
  }
  if ((t & 63) == 0) sh_key[t >> 6] = key;
  __syncthreads();
  key = sh_key[0];
  for (int w = 1; w < 4; w++) key = sh_key[w] > key ? sh_key[w] : key;
  const int best = 0xffff - (int)(key & 0xffff);  // the root is always accepted, so key != 0
  const int L = (int)(key >> 16) - 1;
  if (t == best) {
#pragma unroll
    for (int w = 0; w < kAncWords; w++) sh_best[w] = my[w];
  }
  __syncthreads();
  const int stride = max_depth + 1;
  if (t < N && ((sh_best[t >> 5] >> (t & 31)) & 1u)) {
    path[b * stride + depth] = t;
    tok_user[b * stride + depth] = a;
  }
  if (t > L && t < stride) {
    path[b * stride + t] = -1;
    tok_user[b * stride + t] = -1;
  }
  if (t == 0) {
    len_ctx[b] = L;
    len_user[b] = L;
  }
}

hipError_t launch_accept(hipStream_t st, int batch, const SeqMeta& meta, const int32_t* parent,
                         const int32_t* tokens, int32_t* status, const ArgmaxPartial* partial,
                         int nchunks, int max_depth, int32_t* argmax_out, int32_t* path,
                         int32_t* len_ctx, int32_t* len_user, int32_t* tok_user) {
  hipLaunchKernelGGL(k_accept, dim3(batch), dim3(256), 0, st, meta, parent, tokens, status, partial, nchunks,
                     max_depth, argmax_out, path, len_ctx, len_user, tok_user);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// KV compaction: slot S+j <- slot S+path[j], j = 1..L, for K and V of every kv head and layer.
// path[j] >= j and the path is increasing, so slot S+j can be the source of an earlier step.  One
// thread owns one 16-byte column (layer, K|V, head, offset in the row) and walks j upwards: every
// read of a slot happens before the same thread overwrites it, and no other thread touches the column.
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
  const int S = meta.kv_len[b];
  int L = acc_len[b];
  L = L < 0 ? 0 : (L > max_depth ? max_depth : L);
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) new_len[b] = S + L + 1;
  const int col = blockIdx.x * 256 + threadIdx.x;
  if (col >= Hkv * row_vecs) return;
  const int h = col / row_vecs, vec = col - h * row_vecs;
  char* base = reinterpret_cast<char*>(which ? ptrs.v[layer] : ptrs.k[layer]);
  const int N = meta.node_off[b + 1] - meta.node_off[b];
  for (int j = 1; j <= L; j++) {
    int src = path[b * (max_depth + 1) + j];
    if (src == j) continue;
    if (src < j || src >= N) continue;  // cannot happen for a path produced by k_accept
    const int64_t so = slot_offset(geo, b, S + src, h), doff = slot_offset(geo, b, S + j, h);
    const uint4 x = *reinterpret_cast<const uint4*>(base + (so << elem_shift) + (int64_t)vec * 16);
    *reinterpret_cast<uint4*>(base + (doff << elem_shift) + (int64_t)vec * 16) = x;
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

// Scalar (non-MFMA) tree attention and the split merge.  This is the fp32 path (all arithmetic in
// fp32, accurate expf) and the fallback for shapes the MFMA kernel does not take.  gfx950 only.
//
// Tree attention, Section 3.2 of the paper: node i of a tree attends to the KV-cached prefix
// (slots 0..S-1) and to the tree nodes on its own ancestor chain (slots S+a, a in anc(i)).
#include "cb_internal.h"

namespace cb {

__device__ __forceinline__ float ld_elem(const float* p) { return *p; }
__device__ __forceinline__ float ld_elem(const uint16_t* p) { return __uint_as_float(((uint32_t)*p) << 16); }

__device__ __forceinline__ void st_elem(float* p, float x) { *p = x; }
__device__ __forceinline__ void st_elem(uint16_t* p, float x) {  // round to nearest even
  uint32_t u = __float_as_uint(x);
  u += 0x7fffu + ((u >> 16) & 1u);
  *p = (uint16_t)(u >> 16);
}

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) x = fmaxf(x, __shfl_xor(x, s, 64));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) x += __shfl_xor(x, s, 64);
  return x;
}

template <typename T, int D>
__device__ __forceinline__ float dot_row(const float* __restrict__ sq, const T* __restrict__ krow) {
  constexpr int VEC = 16 / sizeof(T);
  float s = 0.f;
#pragma unroll
  for (int v = 0; v < D / VEC; v++) {
    const uint4 u = reinterpret_cast<const uint4*>(krow)[v];
    if constexpr (sizeof(T) == 2) {
      const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
      for (int k = 0; k < 4; k++) {
        s = fmaf(sq[v * 8 + 2 * k], __uint_as_float(w[k] << 16), s);
        s = fmaf(sq[v * 8 + 2 * k + 1], __uint_as_float(w[k] & 0xffff0000u), s);
      }
    } else {
      s = fmaf(sq[v * 4 + 0], __uint_as_float(u.x), s);
      s = fmaf(sq[v * 4 + 1], __uint_as_float(u.y), s);
      s = fmaf(sq[v * 4 + 2], __uint_as_float(u.z), s);
      s = fmaf(sq[v * 4 + 3], __uint_as_float(u.w), s);
    }
  }
  return s;
}

constexpr int kSimtTile = 1024;  // keys whose scores are held in LDS at a time

// grid: x = node * Hq + head (node local to the sequence), y = split, z = sequence
template <typename T, int D>
__global__ __launch_bounds__(256) void k_attn_simt(AttnParams p, SeqMeta meta) {
  __shared__ float sq[D];
  __shared__ float ss[kSimtTile];
  __shared__ float red[4];
  __shared__ float sacc[256];
  __shared__ uint32_t sanc[kAncWords];
  const int b = blockIdx.z, tid = threadIdx.x;
  const int off = meta.node_off[b];
  const int N = meta.node_off[b + 1] - off;
  const int S = meta.kv_len[b];
  const int i = blockIdx.x / p.Hq, h = blockIdx.x - i * p.Hq;  // (rows on x: up to 256 nodes x 1024 heads)
  if (i >= N) return;
  const int len = S + N;
  const int k0 = blockIdx.y * p.chunk;
  if (k0 >= len) return;
  const int k1 = (k0 + p.chunk < len) ? k0 + p.chunk : len;
  const int nsplit_b = (len + p.chunk - 1) / p.chunk;
  const int hk = h / (p.Hq / p.Hkv);
  const T* qrow = reinterpret_cast<const T*>(p.q) + ((int64_t)(off + i) * p.Hq + h) * D;
  if (tid < D) sq[tid] = ld_elem(qrow + tid);
  if (tid < kAncWords) sanc[tid] = p.anc[(int64_t)(off + i) * kAncWords + tid];
  __syncthreads();
  const T* kbase = reinterpret_cast<const T*>(p.kv.k);
  const T* vbase = reinterpret_cast<const T*>(p.kv.v);
  constexpr int NS = 256 / D;  // key slices that accumulate V in parallel
  const int d = tid % D, slice = tid / D;
  float m_run = -INFINITY, l_run = 0.f, acc = 0.f;
  for (int t0 = k0; t0 < k1; t0 += kSimtTile) {
    const int tl = (k1 - t0 < kSimtTile) ? k1 - t0 : kSimtTile;
    float mloc = -INFINITY;
    for (int jj = tid; jj < tl; jj += 256) {
      const int key = t0 + jj;
      const bool vis = key < S || ((sanc[(key - S) >> 5] >> ((key - S) & 31)) & 1u);
      float s = -INFINITY;
      if (vis) s = p.scale * dot_row<T, D>(sq, kbase + slot_offset(p.kv, b, key, hk));
      ss[jj] = s;
      mloc = fmaxf(mloc, s);
    }
    mloc = wave_max(mloc);
    __syncthreads();  // also orders the previous tile's reads of ss/red before these writes
    if ((tid & 63) == 0) red[tid >> 6] = mloc;
    __syncthreads();
    const float m_tile = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    if (m_tile == -INFINITY) continue;  // nothing visible in this tile (uniform for the workgroup)
    const float m_new = fmaxf(m_run, m_tile);
    float lloc = 0.f;
    for (int jj = tid; jj < tl; jj += 256) {
      const float s = ss[jj];
      const float e = (s == -INFINITY) ? 0.f : expf(s - m_new);
      ss[jj] = e;
      lloc += e;
    }
    lloc = wave_sum(lloc);
    if ((tid & 63) == 0) red[tid >> 6] = lloc;
    __syncthreads();
    const float l_tile = red[0] + red[1] + red[2] + red[3];
    const float alpha = (m_run == -INFINITY) ? 0.f : expf(m_run - m_new);
    l_run = l_run * alpha + l_tile;
    acc *= alpha;
    // eight independent V loads in flight per thread (masked keys carry weight 0 and read slot t0)
    for (int j0 = slice; j0 < tl; j0 += 8 * NS) {
      float e[8], x[8];
#pragma unroll
      for (int u = 0; u < 8; u++) {
        const int jj = j0 + u * NS;
        e[u] = jj < tl ? ss[jj] : 0.f;
        const int key = (e[u] != 0.f) ? t0 + jj : t0;
        x[u] = ld_elem(vbase + slot_offset(p.kv, b, key, hk) + d);
      }
#pragma unroll
      for (int u = 0; u < 8; u++) acc = fmaf(e[u], x[u], acc);
    }
    m_run = m_new;
    __syncthreads();
  }
  sacc[tid] = acc;
  __syncthreads();
  if (tid < D) {
    float o = 0.f;
#pragma unroll
    for (int s = 0; s < NS; s++) o += sacc[s * D + tid];
    const int64_t row = (int64_t)(off + i) * p.Hq + h;
    if (nsplit_b == 1) {
      st_elem(reinterpret_cast<T*>(p.out) + row * D + tid, o / l_run);
    } else {
      float* pr = p.partial + (row * p.nsplit + blockIdx.y) * partial_stride(D);
      pr[tid] = o;
      if (tid == 0) { pr[D] = m_run; pr[D + 1] = l_run; }
    }
  }
}

hipError_t launch_attn_simt(hipStream_t st, const AttnParams& p, const SeqMeta& meta, int dtype,
                            int max_nodes_in_call) {
  dim3 grid(max_nodes_in_call * p.Hq, p.nsplit, p.batch);
  dim3 block(256);
  if (dtype == CB_F32 && p.D == 64) hipLaunchKernelGGL((k_attn_simt<float, 64>), grid, block, 0, st, p, meta);
  else if (dtype == CB_F32 && p.D == 128) hipLaunchKernelGGL((k_attn_simt<float, 128>), grid, block, 0, st, p, meta);
  else if (dtype == CB_BF16 && p.D == 64) hipLaunchKernelGGL((k_attn_simt<uint16_t, 64>), grid, block, 0, st, p, meta);
  else if (dtype == CB_BF16 && p.D == 128) hipLaunchKernelGGL((k_attn_simt<uint16_t, 128>), grid, block, 0, st, p, meta);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

// Merge of the split partials: m = max m_t, l = sum l_t e^(m_t - m), o = sum o_t e^(m_t - m) / l.
// A split that saw no visible key carries m_t = -inf, l_t = 0 and contributes nothing.
// grid: x = global row (node * Hq + head); block = D threads.  Rows of single-split sequences were
// already finished by the attention kernel.
template <typename T, int D>
__global__ __launch_bounds__(D) void k_merge(AttnParams p, SeqMeta meta) {
  const int64_t row = blockIdx.x;
  const int node = (int)(row / p.Hq);
  int b = 0;
  while (b + 1 < p.batch && node >= meta.node_off[b + 1]) b++;
  const int len = meta.kv_len[b] + (meta.node_off[b + 1] - meta.node_off[b]);
  const int ns = (len + p.chunk - 1) / p.chunk;
  if (ns <= 1) return;
  constexpr int PS = partial_stride(D);
  const float* pr = p.partial + row * p.nsplit * PS;
  float m = -INFINITY;
  for (int t = 0; t < ns; t++) m = fmaxf(m, pr[t * PS + D]);
  float l = 0.f, o = 0.f;
  for (int t = 0; t < ns; t++) {
    const float mt = pr[t * PS + D];
    const float w = (mt == -INFINITY) ? 0.f : expf(mt - m);
    l = fmaf(pr[t * PS + D + 1], w, l);
    o = fmaf(pr[t * PS + threadIdx.x], w, o);
  }
  st_elem(reinterpret_cast<T*>(p.out) + row * D + threadIdx.x, o / l);
}

hipError_t launch_merge(hipStream_t st, const AttnParams& p, const SeqMeta& meta, int dtype, int total_nodes) {
  dim3 grid(total_nodes * p.Hq);
  if (dtype == CB_F32 && p.D == 64) hipLaunchKernelGGL((k_merge<float, 64>), grid, dim3(64), 0, st, p, meta);
  else if (dtype == CB_F32 && p.D == 128) hipLaunchKernelGGL((k_merge<float, 128>), grid, dim3(128), 0, st, p, meta);
  else if (dtype == CB_BF16 && p.D == 64) hipLaunchKernelGGL((k_merge<uint16_t, 64>), grid, dim3(64), 0, st, p, meta);
  else if (dtype == CB_BF16 && p.D == 128) hipLaunchKernelGGL((k_merge<uint16_t, 128>), grid, dim3(128), 0, st, p, meta);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace cb

// Device code of the greedy acceptance check (Section 3.2 of the paper, last paragraphs): the
// vocabulary argmax of every tree node's logits row, and the longest accepted root-to-leaf path.
// Shared by the stand-alone argmax / acceptance kernels and by the attention kernel, whose
// workgroups can run this work once their own attention duty is over.  gfx950 only.
#pragma once
#include "cb_internal.h"

namespace cb {

// Every pointer these functions are handed is device (global) memory, but it reaches them as a
// generic pointer inside an argument struct.  Accesses through a generic pointer are flat
// instructions, which the compiler orders behind every outstanding LDS-DMA load (they might touch
// LDS) -- a vmcnt(0) wait in the middle of the attention kernel's ring.  So each access site casts
// to the global address space.
#define CBL_GLOBAL __attribute__((address_space(1)))
template <typename T>
__device__ __forceinline__ CBL_GLOBAL T* as_global(T* p) {
  return (CBL_GLOBAL T*)p;
}

__device__ __forceinline__ float elem_to_float(float x) { return x; }
__device__ __forceinline__ float elem_to_float(uint16_t x) { return __uint_as_float(((uint32_t)x) << 16); }

// (value, index) pairs are ordered "larger value, then smaller index" at every level, so equal
// maxima (common with bf16 logits) resolve to the lowest index exactly as a serial scan does.
// Both forms are written with selects: as branches they cost several times more than the loads
// they follow.
__device__ __forceinline__ void amax_take(float& bv, int& bi, float v, int i) {
  const bool take = (v > bv) | ((v == bv) & (i < bi));
  bv = take ? v : bv;
  bi = take ? i : bi;
}
// the same when the candidate's index is known to be larger than the incumbent's
__device__ __forceinline__ void amax_take_later(float& bv, int& bi, float v, int i) {
  const bool take = v > bv;
  bv = take ? v : bv;
  bi = take ? i : bi;
}

// Wave-wide reductions that leave the result in every lane, without LDS traffic: four rotations
// inside each row of 16 lanes (DPP row_ror:1,2,4,8), then the gfx950 row swaps for the four rows
// (v_permlane16_swap exchanges odd rows of one operand with even rows of the other,
// v_permlane32_swap the upper half of one with the lower half of the other).
template <typename Op>
__device__ __forceinline__ uint32_t wave_allreduce_u32(uint32_t x, Op op) {
  x = op(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x121, 0xf, 0xf, false));
  x = op(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x122, 0xf, 0xf, false));
  x = op(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x124, 0xf, 0xf, false));
  x = op(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x128, 0xf, 0xf, false));
  const auto a = __builtin_amdgcn_permlane16_swap(x, x, false, false);
  x = op(a[0], a[1]);
  const auto b = __builtin_amdgcn_permlane32_swap(x, x, false, false);
  return op(b[0], b[1]);
}
__device__ __forceinline__ float wave_max_f32(float x) {
  return __uint_as_float(wave_allreduce_u32(__float_as_uint(x), [](uint32_t p, uint32_t q) {
    return __float_as_uint(fmaxf(__uint_as_float(p), __uint_as_float(q)));
  }));
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t x) {
  return wave_allreduce_u32(x, [](uint32_t p, uint32_t q) { return p < q ? p : q; });
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x) {
  return wave_allreduce_u32(x, [](uint32_t p, uint32_t q) { return p > q ? p : q; });
}
// first maximum over the wave's (value, index) pairs: the largest value, and the smallest index
// among the lanes that hold it (+0 and -0 compare equal, as in a serial scan with '>')
__device__ __forceinline__ void wave_first_max(float& bv, int& bi) {
  const float m = wave_max_f32(bv);
  bi = (int)wave_min_u32(bv == m ? (uint32_t)bi : 0x7fffffffu);
  bv = m;
}

// ArgmaxPartial travels as one 64-bit word so that it can be written and read with single
// agent-scope accesses.
__device__ __forceinline__ unsigned long long amax_pack(float v, int i) {
  return (unsigned long long)__float_as_uint(v) | ((unsigned long long)(uint32_t)i << 32);
}
template <bool COHERENT>
__device__ __forceinline__ void amax_store(ArgmaxPartial* dst, float v, int i) {
  CBL_GLOBAL unsigned long long* p = (CBL_GLOBAL unsigned long long*)dst;
  if (COHERENT) __hip_atomic_store(p, amax_pack(v, i), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else *p = amax_pack(v, i);
}
template <bool COHERENT>
__device__ __forceinline__ void amax_load(const ArgmaxPartial* src, float& v, int& i) {
  const CBL_GLOBAL unsigned long long* p = (const CBL_GLOBAL unsigned long long*)src;
  const unsigned long long x = COHERENT ? __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : *p;
  v = __uint_as_float((uint32_t)x);
  i = (int)(uint32_t)(x >> 32);
}

struct ScanLds {
  float v[8];
  int i[8];
};

// First maximum of elements [c*kArgmaxChunk, min(V, (c+1)*kArgmaxChunk)) of one logits row by a
// workgroup of NT threads, in two halves so that other work can go between the loads and their use:
// issue() requests all of the thread's 16-byte loads at once, consume() reduces them (plus the
// elements a misaligned or ragged row leaves over) to one candidate per wavefront, which lane 0
// of each wave leaves in `sh`.  After a workgroup barrier combine() gives the result (any thread).
template <typename T, int NT>
struct ChunkScan {
  static constexpr int VEC = 16 / sizeof(T);
  static constexpr int kVecPerThread = kArgmaxChunk / VEC / NT;
  static_assert(kVecPerThread >= 1, "chunk smaller than one load per thread");
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4 u[kVecPerThread];
  int64_t start, end, vec_end, nvec;

  // (no __restrict__ on the row: the loads must stay where they are written, in front of the
  // caller's later waits, and not drift down to their first use)
  // UNTRACKED: the loads are issued as instructions the compiler does not know to be loads (it
  // would wait for every LDS-DMA request in flight at their first use); the caller must have
  // waited for them (vmcnt) before pin_here() and consume().
  template <bool UNTRACKED = false>
  __device__ __forceinline__ void issue(const T* base, int64_t V, int c, int tid) {
    start = (int64_t)c * kArgmaxChunk;
    end = (start + kArgmaxChunk < V) ? start + kArgmaxChunk : V;
    const bool aligned = ((reinterpret_cast<uintptr_t>(base + start)) & 15) == 0;
    nvec = aligned ? (end - start) / VEC : 0;
    vec_end = start + nvec * VEC;
    const CBL_GLOBAL u32x4* vp = (const CBL_GLOBAL u32x4*)(base + start);
    if (nvec > 0) {  // (uniform; lanes past the end re-read the last vector and ignore it later, so
                     //  the loads are unconditional and nothing has to wait for them here)
#pragma unroll
      for (int k = 0; k < kVecPerThread; k++) {
        const int64_t i = tid + k * NT;
        if constexpr (UNTRACKED) {
          asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(u[k]) : "v"(vp + (i < nvec ? i : nvec - 1)) : "memory");
        } else {
          u[k] = vp[i < nvec ? i : nvec - 1];
        }
      }
    }
  }

  // Keeps the reduction of the loaded vectors at (or behind) this point of the program: without it
  // the compiler moves that loop-invariant arithmetic, and the wait for the loads with it, to the
  // front of the caller's loop.
  __device__ __forceinline__ void pin_here() {
#pragma unroll
    for (int k = 0; k < kVecPerThread; k++)
      asm volatile("" : "+v"(u[k]));
  }

  __device__ __forceinline__ void consume(const T* base, int tid, ScanLds& sh) {
    float bv = -INFINITY;
    int bi = 0x7fffffff;
#pragma unroll
    for (int k = 0; k < kVecPerThread; k++) {
      const int64_t i = tid + k * NT;
      if (i >= nvec) continue;
      const int e0 = (int)(start + i * VEC);
      if constexpr (sizeof(T) == 2) {
        const uint32_t w[4] = {u[k].x, u[k].y, u[k].z, u[k].w};
#pragma unroll
        for (int j = 0; j < 4; j++) {  // (a thread meets its elements in increasing index order)
          amax_take_later(bv, bi, __uint_as_float(w[j] << 16), e0 + 2 * j);
          amax_take_later(bv, bi, __uint_as_float(w[j] & 0xffff0000u), e0 + 2 * j + 1);
        }
      } else {
        amax_take_later(bv, bi, __uint_as_float(u[k].x), e0);
        amax_take_later(bv, bi, __uint_as_float(u[k].y), e0 + 1);
        amax_take_later(bv, bi, __uint_as_float(u[k].z), e0 + 2);
        amax_take_later(bv, bi, __uint_as_float(u[k].w), e0 + 3);
      }
    }
    for (int64_t i = vec_end + tid; i < end; i += NT) amax_take_later(bv, bi, elem_to_float(as_global(base)[i]), (int)i);
    wave_first_max(bv, bi);
    if ((tid & 63) == 0) { sh.v[tid >> 6] = bv; sh.i[tid >> 6] = bi; }
  }

  static __device__ __forceinline__ void combine(const ScanLds& sh, float& bv, int& bi) {
    bv = sh.v[0];
    bi = sh.i[0];
#pragma unroll
    for (int w = 1; w < NT / 64; w++) amax_take(bv, bi, sh.v[w], sh.i[w]);
  }
};

// The whole scan in one go; the result is valid in every thread.  The caller separates two calls
// that share `sh` by a barrier.
template <typename T, int NT>
__device__ __forceinline__ void scan_chunk(const T* __restrict__ base, int64_t V, int c, int tid, ScanLds& sh,
                                           float& bv, int& bi) {
  ChunkScan<T, NT> cs;
  cs.issue(base, V, c, tid);
  cs.consume(base, tid, sh);
  __syncthreads();
  ChunkScan<T, NT>::combine(sh, bv, bi);
}

// Greedy acceptance of one sequence's tree by a workgroup of at least 256 threads (thread t owns
// node t).  A node is accepted when every non-root node on its chain carries the token generated at
// that node's parent; with match = {x : tok[x] == a[parent(x)]} (root included) that is anc[c]
// being a subset of match.  The accepted node of greatest depth wins (lowest index among equals);
// its ancestor set *is* the path, each member sitting at position depth(member) = |anc(member)| - 1.
// COHERENT: the argmax partials were written by other workgroups of the same launch (agent-scope
// stores) and are read with agent-scope loads.  Ends with a barrier, so `sh` may be reused at once.
struct AcceptLds {
  int a[CB_MAX_NODES];
  AncScratch anc;
  uint32_t match[kAncWords];
  uint32_t best[kAncWords];
  uint32_t key[4];
};

struct AcceptArgs {
  const int32_t* parent;   // [sumN] local parent indices
  const int32_t* tokens;   // [sumN] draft tokens
  int32_t* status;
  const ArgmaxPartial* partial;  // [sumN][nchunks] entries, `slot_stride` entries apart
  int32_t slot_stride;     // 1: packed.  16: one entry per 128-byte line, for entries that many workgroups
                           // write through to memory at the same time (neighbours would share a line)
  int32_t nchunks;
  int32_t max_depth;
  int32_t* argmax_out;     // [sumN]
  int32_t* path;           // [B][max_depth + 1]
  int32_t* len_ctx;        // [B] (kept for the compaction call)
  int32_t* len_user;       // [B]
  int32_t* tok_user;       // [B][max_depth + 1]
  int32_t* done_flag;      // [B] or null: host-visible words that receive done_value once the sequence's
  int32_t done_value;      // user results are visible to the host (the host form polls them)
};

// Tells a polling host that sequence b's results have arrived.  Called by every thread that wrote
// results, after its stores: the system-scope release fence makes the wave's earlier stores visible
// to the host before the flag store that follows can be.
__device__ __forceinline__ void publish_done(const AcceptArgs& g, int b, bool writer) {
  if (!g.done_flag) return;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "");
  if (writer) __hip_atomic_store(as_global(g.done_flag) + b, g.done_value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

template <bool COHERENT>
__device__ __forceinline__ void accept_sequence(AcceptLds& sh, const AcceptArgs& g, int b, int off, int N) {
  const int t = threadIdx.x;
  N = N > CB_MAX_NODES ? CB_MAX_NODES : N;
  // everything the thread needs from memory is requested before the first use: the node's tree
  // entries, then its row's partial maxima, four at a time
  int par_raw = -1, tok = 0;
  if (t < N) {
    par_raw = as_global(g.parent)[off + t];
    tok = as_global(g.tokens)[off + t];
  }
  int a = -1;
  if (t < N) {
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    const ArgmaxPartial* row = g.partial + (int64_t)(off + t) * g.nchunks * g.slot_stride;
    for (int c0 = 0; c0 < g.nchunks; c0 += 4) {
      float v[4];
      int i[4];
#pragma unroll
      for (int u = 0; u < 4; u++)  // (a repeated entry changes nothing)
        amax_load<COHERENT>(row + (int64_t)(c0 + u < g.nchunks ? c0 + u : g.nchunks - 1) * g.slot_stride, v[u], i[u]);
#pragma unroll
      for (int u = 0; u < 4; u++) amax_take(bv, bi, v[u], i[u]);
    }
    a = bi;
    as_global(g.argmax_out)[off + t] = a;
  }
  if (t < CB_MAX_NODES) sh.a[t] = a;
  __syncthreads();
  bool match = false;
  int par = -1;
  if (t < N) {
    // (the same repair as sanitized_parent(): entries outside [0, t) become "child of the root")
    if (t == 0) {
      if (par_raw != -1) __hip_atomic_fetch_or(as_global(g.status), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
      par = par_raw;
      if (par < 0 || par >= t) {
        __hip_atomic_fetch_or(as_global(g.status), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        par = 0;
      }
    }
    match = (t == 0) || (tok == sh.a[par]);
  }
  const int unresolved = build_ancestor_sets(sh.anc, N, par, jump_rounds(g.max_depth));
  const unsigned long long bal = __ballot(match);
  if ((t & 63) == 0 && t < CB_MAX_NODES) {
    sh.match[(t >> 6) * 2] = (uint32_t)bal;
    sh.match[(t >> 6) * 2 + 1] = (uint32_t)(bal >> 32);
  }
  __syncthreads();
  uint32_t my[kAncWords];
  int depth = -1;
  bool acc = t < N;
#pragma unroll
  for (int w = 0; w < kAncWords; w++) {
    my[w] = (t < N) ? sh.anc.anc[t][w] : 0u;
    depth += __popc(my[w]);
    acc = acc && ((my[w] & ~sh.match[w]) == 0u);
  }
  if (depth > g.max_depth || unresolved >= 0) {  // (an unresolved node is deeper than the rounds reach, hence too deep)
    acc = false;
    if (t < N) __hip_atomic_fetch_or(as_global(g.status), 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  uint32_t key = acc ? ((uint32_t)(depth + 1) << 16) | (uint32_t)(0xffff - t) : 0u;
  key = wave_max_u32(key);
  if ((t & 63) == 0 && t < CB_MAX_NODES) sh.key[t >> 6] = key;
  __syncthreads();
  key = sh.key[0];
  for (int w = 1; w < 4; w++) key = sh.key[w] > key ? sh.key[w] : key;
  const int best = 0xffff - (int)(key & 0xffff);  // the root is always accepted, so key != 0
  const int L = (int)(key >> 16) - 1;
  if (t == best) {
#pragma unroll
    for (int w = 0; w < kAncWords; w++) sh.best[w] = my[w];
  }
  __syncthreads();
  const int stride = g.max_depth + 1;
  if (t < N && ((sh.best[t >> 5] >> (t & 31)) & 1u)) {
    as_global(g.path)[b * stride + depth] = t;
    as_global(g.tok_user)[b * stride + depth] = a;
  }
  if (t > L && t < stride) {
    as_global(g.path)[b * stride + t] = -1;
    as_global(g.tok_user)[b * stride + t] = -1;
  }
  if (t == 0) {
    as_global(g.len_ctx)[b] = L;
    as_global(g.len_user)[b] = L;
  }
  if (g.done_flag) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "");  // every wave's result stores, before the barrier
  __syncthreads();
  publish_done(g, b, t == 0);
}

// The same acceptance for a tree of at most 64 nodes by ONE wavefront (lane t owns node t; the
// other waves of the workgroup are not involved and may do something else meanwhile): no LDS
// allocation and no barrier, the ancestor sets are 64-bit lane values combined with lane permutes.
__device__ __forceinline__ unsigned long long shfl_u64(unsigned long long x, int lane) {
  const uint32_t lo = __shfl((uint32_t)x, lane, 64), hi = __shfl((uint32_t)(x >> 32), lane, 64);
  return (unsigned long long)lo | ((unsigned long long)hi << 32);
}
template <bool COHERENT>
__device__ __forceinline__ void accept_wave(const AcceptArgs& g, int b, int off, int N) {
  const int t = threadIdx.x & 63;
  N = N > 64 ? 64 : N;
  const bool live = t < N;
  int par_raw = -1, tok = 0;
  if (live) {
    par_raw = as_global(g.parent)[off + t];
    tok = as_global(g.tokens)[off + t];
  }
  int a = -1;
  if (live) {
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    const ArgmaxPartial* row = g.partial + (int64_t)(off + t) * g.nchunks * g.slot_stride;
    for (int c0 = 0; c0 < g.nchunks; c0 += 4) {
      float v[4];
      int i[4];
#pragma unroll
      for (int u = 0; u < 4; u++)
        amax_load<COHERENT>(row + (int64_t)(c0 + u < g.nchunks ? c0 + u : g.nchunks - 1) * g.slot_stride, v[u], i[u]);
#pragma unroll
      for (int u = 0; u < 4; u++) amax_take(bv, bi, v[u], i[u]);
    }
    a = bi;
    as_global(g.argmax_out)[off + t] = a;
  }
  int par = -1;
  if (live) {
    if (t == 0) {
      if (par_raw != -1) __hip_atomic_fetch_or(as_global(g.status), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
      par = par_raw;
      if (par < 0 || par >= t) {
        __hip_atomic_fetch_or(as_global(g.status), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        par = 0;
      }
    }
  }
  const int a_par = __shfl(a, par < 0 ? 0 : par, 64);
  const bool match = live && (t == 0 || tok == a_par);
  const unsigned long long matched = __ballot(match);
  unsigned long long mine = live ? (1ull << t) : 0ull;
  int j = par;
  const int rounds = jump_rounds(g.max_depth);
  for (int r = 0; r < rounds && r < 6; r++) {  // six rounds complete any tree of 64 nodes
    const int src = j < 0 ? 0 : j;
    const unsigned long long other = shfl_u64(mine, src);
    const int jj = __shfl(j, src, 64);
    if (j >= 0) {
      mine |= other;
      j = jj;
    }
  }
  const int depth = __popcll(mine) - 1;
  bool acc = live && (mine & ~matched) == 0ull;
  if (live && (depth > g.max_depth || j >= 0)) {
    acc = false;
    __hip_atomic_fetch_or(as_global(g.status), 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  uint32_t key = acc ? ((uint32_t)(depth + 1) << 16) | (uint32_t)(0xffff - t) : 0u;
  key = wave_max_u32(key);
  const int best = 0xffff - (int)(key & 0xffff);  // the root is always accepted, so key != 0
  const int L = (int)(key >> 16) - 1;
  const unsigned long long on_path = shfl_u64(mine, best);
  const int stride = g.max_depth + 1;
  if (live && ((on_path >> t) & 1ull)) {
    as_global(g.path)[b * stride + depth] = t;
    as_global(g.tok_user)[b * stride + depth] = a;
  }
  for (int d = t; d < stride; d += 64) {
    if (d > L) {
      as_global(g.path)[b * stride + d] = -1;
      as_global(g.tok_user)[b * stride + d] = -1;
    }
  }
  if (t == 0) {
    as_global(g.len_ctx)[b] = L;
    as_global(g.len_user)[b] = L;
  }
  publish_done(g, b, t == 0);
}

// The logits work of one verification call as a list of items (row, chunk), item = row * nchunks +
// chunk, shared out among the workgroups of a launch that has at least as many workgroups as there
// are items: workgroup w takes item w.  bf16 logits and sequences of at most 64 nodes only (the
// launcher checks all three).
struct LogitsWork {
  const uint16_t* logits;  // [rows][V] bf16
  int64_t V;
  int32_t rows;         // total tree nodes of the call
  int32_t batch;
  ArgmaxPartial* partial_out;  // same memory and spacing as accept.partial
  uint32_t* tickets;    // [B] items finished per sequence, zero between launches
  AcceptArgs accept;
};

struct TailLds {
  ScanLds scan;
  int flag0;
};

// A workgroup's item in steps that the attention code calls where they cost least: the loads in
// front of its first K/V requests (prefetch_first), the reduction once they have landed
// (mid_consume), the combination of the waves' candidates and the partial's store behind the next
// barrier (mid_combine), the ticket once a full wait has covered that store (early_ticket); what has
// not happened by the end of the key sweep is caught up on there (scan_first and the ticket halves,
// beside the attention's own stores and ticket).  The ticket counts the finished items of the
// item's sequence; the workgroup whose ticket completes the count (every partial is then in memory:
// each workgroup waited for its own agent-scope store first) has its first wave run the acceptance
// for that sequence (accept_first).  Nobody waits for anybody, so the order in which workgroups run
// is irrelevant.  finish() does whatever has not been done by then (a workgroup may leave the
// attention early).  Every method except the ticket halves must be called by all NT threads.
template <int NT>
struct LogitsHook {
  const LogitsWork& lw;
  const SeqMetaLanes& ml;  // the sequences' shapes, one per lane (no memory access when they are looked up)
  TailLds& sh;
  int wg;
  int state;  // 0 untouched, 1 partial stored but not counted, 2 no item, 3 counted, 4 loads in flight,
              // 5 the waves' candidates are in LDS (not yet combined), 6 counted and, where it fell to
              // this workgroup, accepted, 7 partial stored and its ticket already drawn (early_old)
  uint32_t early_old = 0;  // thread 0: what the early ticket returned
  int b0;     // the item's sequence
  ChunkScan<uint16_t, NT> pre;
  __attribute__((address_space(3))) unsigned long long* dbg = nullptr;  // timing aid: 8 timestamps (thread 0) in LDS, or null

  __device__ __forceinline__ LogitsHook(const LogitsWork& lw_, const SeqMetaLanes& ml_, TailLds& sh_, int wg_)
      : lw(lw_), ml(ml_), sh(sh_), wg(wg_), state(0), b0(0) {}
  __device__ __forceinline__ int node_off(int b) const { return __builtin_amdgcn_readlane(ml.o0, b); }
  __device__ __forceinline__ int node_count(int b) const { return __builtin_amdgcn_readlane(ml.o1, b) - node_off(b); }
  __device__ __forceinline__ const uint16_t* row_base() const { return lw.logits + (int64_t)(wg / lw.accept.nchunks) * lw.V; }

  __device__ __forceinline__ void stamp(int i) const {  // (timing aid)
    if (dbg != nullptr && threadIdx.x == 0) dbg[i] = wall_clock64();
  }

  // after prefetch_first(): whether every thread has ChunkScan::kVecPerThread loads in flight
  __device__ __forceinline__ bool loads_in_flight() const { return state == 4 && pre.nvec > 0; }
  __device__ __forceinline__ void prefetch_first() {
    if (state != 0) return;
    const int nchunks = lw.accept.nchunks;
    if (wg >= lw.rows * nchunks) {
      state = 2;
      return;
    }
    const int row = wg / nchunks;
    // sequence of the row: the number of sequences that end at or before it
    b0 = __popcll(__ballot((int)(threadIdx.x & 63) < lw.batch - 1 && ml.o1 <= row));
    pre.template issue<true>(row_base(), lw.V, wg - row * nchunks, threadIdx.x);
    state = 4;
  }
  // The scan in pieces, for a caller that has barriers of its own to offer (all threads call each):
  // mid_consume() once the prefetched loads have landed (a vmcnt wait of the caller's that covers
  // them: the compiler does not track them) -- only if the item has no ragged rest,
  // whose loads would have to be waited for on the spot --, a workgroup barrier, mid_combine(), and,
  // once a vmcnt(0) wait of the first wave has followed, early_ticket().  Whatever has not happened
  // by then, scan_first() and the ticket calls below catch up on.
  __device__ __forceinline__ void mid_consume() {
    if (state != 4 || pre.vec_end != pre.end) return;
    pre.pin_here();
    pre.consume(row_base(), threadIdx.x, sh.scan);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the candidate is in LDS before the caller's barrier
    state = 5;
  }
  __device__ __forceinline__ void combine_and_store() {
    if (threadIdx.x == 0) {
      float bv;
      int bi;
      ChunkScan<uint16_t, NT>::combine(sh.scan, bv, bi);
      amax_store<true>(lw.partial_out + (int64_t)wg * lw.accept.slot_stride, bv, bi);
    }
    state = 1;
  }
  __device__ __forceinline__ void mid_combine() {
    if (state == 5) combine_and_store();
  }
  __device__ __forceinline__ void early_ticket() {
    if (state != 1) return;
    if (threadIdx.x == 0)
      early_old = __hip_atomic_fetch_add(as_global(lw.tickets) + b0, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    state = 7;
  }
  __device__ __forceinline__ void scan_first() {
    prefetch_first();
    if (state == 4) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the item's loads (not tracked by the compiler)
      pre.pin_here();
      pre.consume(row_base(), threadIdx.x, sh.scan);
      state = 5;
    }
    if (state != 5) return;
    __syncthreads();  // the waves' candidates are in LDS
    combine_and_store();
  }
  // One thread only -- the one that stored the partial -- after a vmcnt(0) wait that followed
  // scan_first() and before a workgroup barrier.  In two halves so that the caller can put an atomic
  // of its own between them and have both in flight together.
  __device__ __forceinline__ uint32_t ticket_first_issue() const {
    if (state == 7) return early_old;
    return state == 1 ? __hip_atomic_fetch_add(as_global(lw.tickets) + b0, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
  }
  __device__ __forceinline__ void ticket_first_resolve(uint32_t old) {
    if (state != 1 && state != 7) return;
    const uint32_t expect = (uint32_t)node_count(b0) * (uint32_t)lw.accept.nchunks;
    const bool last = old + 1u == expect;
    if (last) __hip_atomic_store(as_global(lw.tickets) + b0, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next launch
    sh.flag0 = last ? 1 : 0;
  }
  // all threads, after the barrier that followed the ticket
  __device__ __forceinline__ void first_counted() {
    if (state == 1 || state == 7) state = 3;
  }
  // all threads, after first_counted(): the acceptance, if this workgroup's ticket completed the
  // sequence -- by the first wave alone, the other waves go on at once
  __device__ __forceinline__ void accept_first() {
    if (state != 3) return;
    if (sh.flag0 && threadIdx.x < 64) accept_wave<true>(lw.accept, b0, node_off(b0), node_count(b0));
    state = 6;
  }

  __device__ __forceinline__ void finish() {
    const bool stamp = dbg != nullptr && threadIdx.x == 0;
    if (stamp) dbg[0] = wall_clock64();
    scan_first();
    if (state == 1 || state == 7) {
      if (threadIdx.x == 0) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        ticket_first_resolve(ticket_first_issue());
      }
      __syncthreads();
      state = 3;
    }
    if (stamp) dbg[1] = wall_clock64();
    accept_first();
    if (stamp) dbg[7] = wall_clock64();
  }
};

}  // namespace cb
